// Device kernels of libeagle (gfx950).  One speculative step = drafting (Sec. 3.1, App. A.1 of the paper),
// tree-masked verification (Sec. 3.3) and acceptance (Sec. 2, App. A.2 Alg. 1) + commit.
#pragma once
#include "common.h"

// ============================================================================ device-side model state
struct TreeDev {
  int M, D;
  int parent[EAGLE_MAX_NODES], depth[EAGLE_MAX_NODES], nchild[EAGLE_MAX_NODES];
  int child[EAGLE_MAX_NODES][EAGLE_MAX_CHILD];           // children in rank order
  unsigned long long anc[EAGLE_MAX_NODES];               // bit u set <=> u is v or an ancestor of v
  int n_level_rows[EAGLE_MAX_DEPTH + 1];                 // level d: depth-d nodes that have children
  int level_rows[EAGLE_MAX_DEPTH + 1][EAGLE_MAX_NODES];
};

struct SeqState {          // all device pointers, one entry per sequence slot
  int* ctx_len;            // positions held by the target KV cache
  int* n_pend;             // target features waiting for the head's first pass (1..D+1)
  int* n_tok;              // committed tokens (= ctx_len + 1 between steps)
  int* step_no;            // draw counter for the generator
  int* commit_base;        // ctx_len before the last commit (read by the compaction kernel)
  int* tokens;             // [max_batch][tok_stride]
  int tok_stride;
};

enum { PASS_VERIFY = 0, PASS_VANILLA, PASS_DRAFT_PENDING, PASS_DRAFT_LEVEL, PASS_PREFILL_T, PASS_PREFILL_D };
struct Pass {
  int kind, rows_per_seq, n_seq, seq0, level, chunk_start, chunk_n;
  // cached target positions of sequences seq0..seq0+3 as the host knows them at launch (it mirrors the device value
  // between calls); saves every kernel a dependent load at its start.  ctx_known = 0: read st.ctx_len instead.
  int ctx_known, ctx0, ctx1, ctx2, ctx3;
};
struct RowInfo {
  int seq, valid, pos, slot, base, rel, node, causal;
  unsigned long long mask;
};

__device__ inline RowInfo row_info(const Pass& p, const TreeDev* t, const SeqState& st, int r) {
  RowInfo o;
  int i = r % p.rows_per_seq;
  o.seq = p.seq0 + r / p.rows_per_seq;
  o.valid = 1; o.causal = 0; o.node = -1; o.mask = 0;
  int ctx;
  if (p.ctx_known) { const int j = o.seq - p.seq0; ctx = j == 0 ? p.ctx0 : j == 1 ? p.ctx1 : j == 2 ? p.ctx2 : p.ctx3; }
  else ctx = st.ctx_len[o.seq];
  switch (p.kind) {
    case PASS_VERIFY:
      o.node = i; o.base = ctx; o.rel = i; o.pos = ctx + t->depth[i]; o.slot = ctx + i; o.mask = t->anc[i];
      break;
    case PASS_VANILLA:
      o.base = ctx; o.rel = 0; o.pos = ctx; o.slot = ctx; o.mask = 1ull;
      break;
    case PASS_DRAFT_PENDING: {
      int np = st.n_pend[o.seq];
      o.valid = i < np;
      o.base = ctx - np; o.rel = o.valid ? i : 0; o.pos = o.base + o.rel; o.slot = o.pos; o.causal = 1;
      o.node = (i == np - 1) ? 0 : -1;
      break;
    }
    case PASS_DRAFT_LEVEL: {
      int v = t->level_rows[p.level][i];
      o.node = v; o.base = ctx - 1; o.rel = v; o.pos = ctx - 1 + t->depth[v]; o.slot = ctx - 1 + v; o.mask = t->anc[v];
      break;
    }
    default:  // PASS_PREFILL_T / PASS_PREFILL_D
      o.valid = i < p.chunk_n;
      o.base = p.chunk_start; o.rel = o.valid ? i : 0; o.pos = o.base + o.rel; o.slot = o.pos; o.causal = 1;
      break;
  }
  return o;
}

struct KVCache {
  void* k; void* v;              // this layer's pages: [phys_page][kv_head][slot_in_page][head_dim]
  const int* page_table;         // [max_batch][pages_per_seq] -> physical page
  int pages_per_seq, page_shift, n_kv_heads, head_dim;
};
__device__ inline size_t kv_offset(const KVCache& c, int seq, int pos, int kvh) {
  int phys = c.page_table[seq * c.pages_per_seq + (pos >> c.page_shift)];
  return (((size_t)phys * c.n_kv_heads + kvh) << c.page_shift | (size_t)(pos & ((1 << c.page_shift) - 1))) * c.head_dim;
}

__device__ inline float cache_load(const float* p) { return *p; }
__device__ inline float cache_load(const bf16_t* p) { return bf16_to_f32(*p); }
__device__ inline void cache_store(float* p, float v) { *p = v; }
__device__ inline void cache_store(bf16_t* p, float v) { *p = f32_to_bf16(v); }

// ============================================================================ block reductions
__device__ inline float wave_sum(float v) {
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ inline float wave_max(float v) {
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
// Sum over the block in a fixed order (wave partials added in wave order): deterministic.
__device__ inline float block_sum(float v, float* sh /*>= 16 floats*/) {
  v = wave_sum(v);
  int w = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) sh[w] = v;
  __syncthreads();
  float t = 0.f;
  for (int i = 0; i < nw; ++i) t += sh[i];
  return t;
}
__device__ inline float block_max(float v, float* sh) {
  v = wave_max(v);
  int w = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) sh[w] = v;
  __syncthreads();
  float t = sh[0];
  for (int i = 1; i < nw; ++i) t = fmaxf(t, sh[i]);
  return t;
}
// (value, index) with the larger value winning and, on equal values, the LOWER index.
__device__ inline void better(float& v, int& i, float v2, int i2) {
  if (v2 > v || (v2 == v && i2 < i)) { v = v2; i = i2; }
}
__device__ inline void block_argmax(float& v, int& i, float* shv, int* shi) {
  for (int o = 32; o > 0; o >>= 1) {
    float v2 = __shfl_xor(v, o, 64);
    int i2 = __shfl_xor(i, o, 64);
    better(v, i, v2, i2);
  }
  int w = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) { shv[w] = v; shi[w] = i; }
  __syncthreads();
  // second level: lanes 0..15 of every wave take one per-wave result each and reduce them with four exchanges (the
  // (value, index) order is total, so the exchange pattern does not matter); lane 0 broadcasts
  const int l = threadIdx.x & 63;
  v = l < nw ? shv[l] : -INFINITY;
  i = l < nw ? shi[l] : 0x7fffffff;
  for (int o = 8; o > 0; o >>= 1) {
    float v2 = __shfl_xor(v, o, 64);
    int i2 = __shfl_xor(i, o, 64);
    better(v, i, v2, i2);
  }
  v = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, v)));
  i = __builtin_amdgcn_readfirstlane(i);
}

// ============================================================================ weight packing
// src: row-major [N][K] (float or bf16).  dst: nplanes packed planes (see wpack_index) of a matrix with KS k-steps;
// plane p starts at dst + p*plane_stride.  Source row n lands in packed row row_offset + map(n):
//   PACK_PLAIN  map(n) = n
//   PACK_ROPE   rows of a head are interleaved so that the two members of a rotate-half pair (i, i + dh/2) become
//               neighbours: head*dh + i + half*dh/2  ->  head*dh + 2i + half
//   PACK_GATE / PACK_UP  fused gate/up matrix: every 32-row block holds gate rows 16j..16j+15 then up rows
//               16j..16j+15, so SwiGLU partners sit in the same block
// One thread builds one 16-byte lane chunk (8 elements along k) of every plane.
enum { PACK_PLAIN = 0, PACK_ROPE = 1, PACK_GATE = 2, PACK_UP = 3 };
__host__ __device__ inline int pack_row_map(int mode, int n, int dh) {
  if (mode == PACK_ROPE) {
    int head = n / dh, r = n % dh, half = dh >> 1;
    return head * dh + 2 * (r % half) + r / half;
  }
  if (mode == PACK_GATE) return (n >> 4) * 32 + (n & 15);
  if (mode == PACK_UP) return (n >> 4) * 32 + 16 + (n & 15);
  return n;
}
template <typename SrcT>
__global__ __launch_bounds__(256) void k_pack_weight(const SrcT* __restrict__ src, bf16_t* __restrict__ dst, int N, int K,
                                                     int row_offset, int KS, int nplanes, size_t plane_stride, int mode, int dh,
                                                     size_t ldn = 0 /*source stride between rows n (0 = K)*/, size_t ldk = 1 /*between columns k*/) {
  if (ldn == 0) ldn = (size_t)K;
  size_t gid = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  int nrb = (N + 31) >> 5;
  size_t total = (size_t)nrb * KS * 64;
  if (gid >= total) return;
  int lane = gid & 63;
  size_t tile = gid >> 6;
  int ks = tile % KS;
  int rb = tile / KS;
  int n = rb * 32 + (lane & 31);
  int k0 = ks * 16 + (lane >> 5) * 8;
  if (n >= N && mode != PACK_PLAIN) return;               // only the plain map pads its last block with zero rows
  bf16_t out[3][8];
  for (int t = 0; t < 8; ++t) {
    float x = 0.f;
    if (n < N && k0 + t < K) {
      if constexpr (sizeof(SrcT) == 4) x = ((const float*)src)[(size_t)n * ldn + (size_t)(k0 + t) * ldk];
      else x = bf16_to_f32(((const bf16_t*)src)[(size_t)n * ldn + (size_t)(k0 + t) * ldk]);
    }
    bf16_t p[3];
    split_bf16(x, p, nplanes);
    for (int q = 0; q < nplanes; ++q) out[q][t] = p[q];
  }
  size_t o = wpack_index(row_offset + pack_row_map(mode, n, dh), k0, KS);
  for (int q = 0; q < nplanes; ++q) {
    u32x4 v;
    v.x = out[q][0] | ((uint32_t)out[q][1] << 16); v.y = out[q][2] | ((uint32_t)out[q][3] << 16);
    v.z = out[q][4] | ((uint32_t)out[q][5] << 16); v.w = out[q][6] | ((uint32_t)out[q][7] << 16);
    *(u32x4*)(dst + q * plane_stride + o) = v;
  }
}

// ---- 4-bit weights (Sec. 4.2: the int4 case study) ---------------------------------------------------------------------
// Weight-only, symmetric, groups of 128 input columns: s = bf16(max|w| / 7), code = clip(rint(w / s), -8, 7) + 8, value
// s * (code - 8).  Layout: "super-tiles" of 32 rows x 64 k = 1 KiB, tile (rb, T) at ((rb*KT + T) * 64) 16-byte lane
// chunks (KT = K / 64); lane l (row l%32, k-half l/32) holds four 32-bit words, word j = the 8 codes of k-step j of
// the super-tile, k = 64T + 16j + 8(l/32) + e, with code e at bit 4*(e/2) + 16*(e%2): ((word >> 4p) & 0x000F000F) |
// 0x43004300 is then the bf16 pair (128 + code 2p, 128 + code 2p+1), i.e. the MFMA A operand of the k-step comes out of
// one shift and one and-or per pair (128 + c is exact in bf16; the offset 136 = 128 + 8 is taken off per group).
// Scales: bf16 [rb][group][lane-half][16] in accumulator-register order: entry (hh, r) belongs to row
// 8*(r/4) + 4*hh + r%4 of the block, so a lane reads the scales of its 16 accumulator rows as 32 contiguous bytes.
#define EAGLE_Q4_GROUP 128
template <typename SrcT>
__global__ __launch_bounds__(256) void k_pack_weight_q4(const SrcT* __restrict__ src, uint32_t* __restrict__ dst, bf16_t* __restrict__ sc,
                                                        int N, int K, int row_offset, int mode, int dh) {
  const int NG = K / EAGLE_Q4_GROUP, KT = K / 64;
  const size_t gid = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int nrows = mode == PACK_PLAIN ? (N + 31) / 32 * 32 : N;          // only the plain map pads its last block
  if (gid >= (size_t)nrows * NG) return;
  const int n = (int)(gid / NG), g = (int)(gid % NG);
  float w[EAGLE_Q4_GROUP];
  float mx = 0.f;
  for (int t = 0; t < EAGLE_Q4_GROUP; ++t) {
    float x = 0.f;
    if (n < N) {
      if constexpr (sizeof(SrcT) == 4) x = ((const float*)src)[(size_t)n * K + g * EAGLE_Q4_GROUP + t];
      else x = bf16_to_f32(((const bf16_t*)src)[(size_t)n * K + g * EAGLE_Q4_GROUP + t]);
    }
    w[t] = x;
    mx = fmaxf(mx, fabsf(x));
  }
  const bf16_t sb = f32_to_bf16(mx / 7.0f);
  const float s = bf16_to_f32(sb), safe = s > 0.f ? s : 1.0f;
  const int prow = row_offset + pack_row_map(mode, n, dh);
  const int rb = prow >> 5, rho = prow & 31, hh = (rho >> 2) & 1, r = 4 * (rho >> 3) + (rho & 3);
  sc[(((size_t)rb * NG + g) * 2 + hh) * 16 + r] = sb;
  for (int st = 0; st < 2; ++st) {                                        // the group's two super-tiles
    const int T = 2 * g + st;
    for (int kh = 0; kh < 2; ++kh) {
      uint32_t words[4];
      for (int j = 0; j < 4; ++j) {
        uint32_t wd = 0;
        for (int e = 0; e < 8; ++e) {
          const float q = fminf(fmaxf(rintf(w[64 * st + 16 * j + 8 * kh + e] / safe), -8.f), 7.f);
          wd |= (uint32_t)((int)q + 8) << (4 * (e >> 1) + 16 * (e & 1));
        }
        words[j] = wd;
      }
      u32x4 v; v.x = words[0]; v.y = words[1]; v.z = words[2]; v.w = words[3];
      *(u32x4*)(dst + (((size_t)rb * KT + T) * 64 + rho + 32 * kh) * 4) = v;
    }
  }
}

// ============================================================================ skinny weight-streaming GEMM
// PT[s][m][n] = sum over the split's k range of W[n][k] * X[m][k];  W packed (NWP bf16 planes), X in XF layout
// (NXP bf16 planes, MT 32-row tiles).  A block is 4 waves; wave w owns row-block blockIdx.x*4+w (32 rows of W)
// and streams it once: every tile is one coalesced 1 KiB load that goes straight into the MFMA A operand.  The
// block's X slice passes through LDS (already in B-operand order) in chunks of CH k-steps.  While a chunk is being
// multiplied, the next chunk's weight tiles AND activation tiles are already on their way into registers, so neither
// HBM nor L2 latency is exposed between chunks.  Products kept: plane pairs (p, q) with p + q < max(NWP, NXP);
// pieces beyond that are below fp32 resolution of the sum.
template <int NXP> struct GemmChunk { static constexpr int CH = NXP == 2 ? 8 : 4; };   // k-steps per LDS stage
template <int NWP, int NXP, int MT>
__global__ __launch_bounds__(256) void k_gemm(const bf16_t* __restrict__ Wp, size_t w_plane_stride,
                                              const bf16_t* __restrict__ XF, float* __restrict__ PT, int NRB, int KS,
                                              int ks_per_split, int Npad) {
  constexpr int CH = GemmChunk<NXP>::CH;
  constexpr int XT = NXP * MT * CH;                             // activation tiles (1 KiB each) per chunk
  constexpr int XR = (XT * 64 + 255) / 256;                     // 16-byte pieces of them per thread
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  u32x4* xs = (u32x4*)smem;                                     // [NXP*MT][CH][64] 16-byte lane chunks
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int rb = min(blockIdx.x * 4 + wave, NRB - 1);           // waves past the end repeat the last block, store nothing
  const bool live = blockIdx.x * 4 + wave < NRB;
  const int s = blockIdx.y;
  const int k_begin = s * ks_per_split;
  const int k_end = min(KS, k_begin + ks_per_split);
  constexpr int PMAX = NWP > NXP ? NWP : NXP;
  f32x16 acc[MT];
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int j = 0; j < 16; ++j) acc[i][j] = 0.f;
  if (k_end <= k_begin) return;
  const int klast = k_end - 1;
  const u32x4* wbase = (const u32x4*)(Wp + (size_t)rb * KS * 512) + lane;

  u32x4 xr[XR], ar[CH][NWP];
  // piece i of a chunk: tile pm = i / (CH*64), k-step kk = (i / 64) % CH, lane-chunk i % 64 (the LDS order)
  auto load_x = [&](int c0) {
#pragma unroll
    for (int u = 0; u < XR; ++u) {
      const int i = min(u * 256 + (int)threadIdx.x, XT * 64 - 1);
      const int pm = i / (CH * 64), kk = (i / 64) % CH, l = i & 63;
      xr[u] = *((const u32x4*)(XF + ((size_t)pm * KS + min(c0 + kk, klast)) * 512) + l);
    }
  };
  auto load_a = [&](int c0) {
#pragma unroll
    for (int u = 0; u < CH; ++u)
#pragma unroll
      for (int p = 0; p < NWP; ++p)
        ar[u][p] = *(const u32x4*)((const bf16_t*)(wbase + (size_t)min(c0 + u, klast) * 64) + p * w_plane_stride);
  };
  auto store_x = [&]() {
#pragma unroll
    for (int u = 0; u < XR; ++u) {
      const int i = u * 256 + (int)threadIdx.x;
      if (i < XT * 64) xs[i] = xr[u];
    }
  };
  load_x(k_begin);
  load_a(k_begin);
  store_x();
  __syncthreads();
  for (int c0 = k_begin; c0 < k_end; c0 += CH) {
    const int nk = min(CH, k_end - c0);
    const bool more = c0 + CH < k_end;
    u32x4 a[CH][NWP];
#pragma unroll
    for (int u = 0; u < CH; ++u)
#pragma unroll
      for (int p = 0; p < NWP; ++p) a[u][p] = ar[u][p];
    if (more) { load_x(c0 + CH); load_a(c0 + CH); }            // in flight while this chunk is multiplied
#pragma unroll
    for (int u = 0; u < CH; ++u) {
      if (u < nk) {
#pragma unroll
        for (int q = 0; q < NXP; ++q)
#pragma unroll
          for (int mt = 0; mt < MT; ++mt) {
            const u32x4 b = xs[((size_t)(q * MT + mt) * CH + u) * 64 + lane];
#pragma unroll
            for (int p = 0; p < NWP; ++p)
              if (p + q < PMAX)
                acc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a[u][p]),
                                                                  __builtin_bit_cast(bf16x8, b), acc[mt], 0, 0, 0);
          }
      }
    }
    __syncthreads();                                            // every wave is done with this chunk's LDS
    if (more) { store_x(); __syncthreads(); }
  }
  if (live) {
    // accumulator register r of lane l holds W-row 8*(r/4) + 4*(l/32) + r%4, X-row l%32; partials are stored
    // PT[s][m][n] (n fastest, which is how every epilogue kernel walks them): registers 4i..4i+3 are 16 contiguous bytes
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      float* out = PT + ((size_t)s * (MT * 32) + mt * 32 + (lane & 31)) * Npad + (size_t)rb * 32 + 4 * (lane >> 5);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        f32x4 v; v.x = acc[mt][4 * i]; v.y = acc[mt][4 * i + 1]; v.z = acc[mt][4 * i + 2]; v.w = acc[mt][4 * i + 3];
        *(f32x4*)(out + 8 * i) = v;
      }
    }
  }
}

// ============================================================================ large-M GEMM (prompt passes of up to 512 rows)
// Same operands and the same PT[s][m][n] result as k_gemm, for passes whose rows fill several 128-row tiles: here the
// MFMA pipes, not the weight stream, are the bound (Sec. 3.1: the head consumes the whole prompt's features, so the
// prompt runs through the target and the head once, as one large matrix product per weight matrix).
//   work-group tile  256 weight rows (8 row blocks) x 128 activation rows (4 row tiles), 4 waves;
//   wave w           row blocks 2w, 2w+1 x all 4 activation tiles: 8 accumulator tiles, 16 MFMAs per k-step
//   activations      the tile's 2 planes x 4 row tiles pass through LDS in chunks of CH k-steps, double-buffered; the
//                    next chunk travels global -> registers while the current one is multiplied (one barrier a chunk)
//   weights          each wave streams its own two row blocks global -> registers one chunk ahead
// Work-groups that share a weight tile (the activation-row tiles of one weight-row tile) get ids 8 apart, i.e. the same
// XCD under round-robin dispatch, next to each other in dispatch order: the tile comes from HBM once and from that
// XCD's L2 afterwards.
__device__ inline void xf_store8(bf16_t* XF, int m, int k8, int MT, int KS, int nplanes, const float* x);   // defined with the row producers below
// SWIGLU (only with S = 1, gate/up matrices): instead of PT the kernel writes silu(gate) * up as the next GEMM's input
// (XF layout, `act`, rows beyond M as zeros).  A row block of the fused matrix holds 16 gate rows and the 16 up rows of
// the same features, and accumulator registers r and r + 8 of a lane are such a pair; the two lanes of an activation
// row swap four values so that each holds 8 consecutive features = its 16 bytes of the output tile.
template <int NXP, bool SWIGLU = false>
__global__ __launch_bounds__(256, 2) void k_gemm_pf(const bf16_t* __restrict__ Wp, const bf16_t* __restrict__ XF,
                                                 float* __restrict__ PT, int NRB, int KS, int ks_per_split, int S, int Npad,
                                                 int MT /*32-row tiles of the pass*/, bf16_t* act = nullptr, int M = 0) {
  constexpr int CH = 4;                                         // k-steps per LDS stage
  constexpr int XT = NXP * 4 * CH;                              // activation tiles (1 KiB) per stage
  constexpr int XR = XT / CH;                                   // activation tiles per stage and k-step = loads per wave and stage
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  u32x4* xs = (u32x4*)smem;                                     // [2 stages][NXP*4 tiles][CH][64]
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int MQ = (MT + 3) >> 2, NT = (NRB + 7) >> 3, G = NT * S;
  // id -> (group = (weight-row tile, split), activation-row tile)
  const int L = blockIdx.x, blk = L / (8 * MQ), rem = L % (8 * MQ), mq = rem >> 3, g = blk * 8 + (rem & 7);
  if (g >= G) return;
  const int nt = g / S, s = g % S;
  const int rbA = min(nt * 8 + 2 * wave, NRB - 1), rbB = min(nt * 8 + 2 * wave + 1, NRB - 1);
  const bool liveA = nt * 8 + 2 * wave < NRB, liveB = nt * 8 + 2 * wave + 1 < NRB;
  const int k_begin = s * ks_per_split, k_end = min(KS, k_begin + ks_per_split);
  if (k_end <= k_begin) return;
  const int klast = k_end - 1;
  f32x16 acc[2][4];
#pragma unroll
  for (int j = 0; j < 2; ++j)
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[j][t][r] = 0.f;
  const u32x4* wA = (const u32x4*)(Wp + (size_t)rbA * KS * 512) + lane;
  const u32x4* wB = (const u32x4*)(Wp + (size_t)rbB * KS * 512) + lane;
  u32x4 xr[XR], ar[CH][2];
  // Activations: global -> registers at the start of a stage, registers -> LDS at its end (the loads have the whole
  // stage to arrive).  Load u of wave w carries tile u (= plane * 4 + row tile) of k-step c0 + w, which is piece
  // (u * CH + w) * 64 + lane of the stage.  Every k range is a multiple of CH (host).
  auto load_x = [&](int c0) {
#pragma unroll
    for (int u = 0; u < XR; ++u) {
      const int plane = u >> 2, mt = min(mq * 4 + (u & 3), MT - 1);
      xr[u] = *((const u32x4*)(XF + (((size_t)plane * MT + mt) * KS + min(c0 + wave, klast)) * 512) + lane);
    }
  };
  auto store_x = [&](int stage) {
#pragma unroll
    for (int u = 0; u < XR; ++u) xs[(size_t)stage * XT * 64 + (size_t)(u * CH + wave) * 64 + lane] = xr[u];
  };
  auto load_a = [&](int c0) {
#pragma unroll
    for (int u = 0; u < CH; ++u) {
      const size_t ko = (size_t)min(c0 + u, klast) * 64;
      ar[u][0] = wA[ko]; ar[u][1] = wB[ko];
    }
  };
  load_x(k_begin);
  load_a(k_begin);
  store_x(0);
  __syncthreads();
  int stage = 0;
  for (int c0 = k_begin; c0 < k_end; c0 += CH, stage ^= 1) {
    // the next stage's activations, in flight while this stage is multiplied (issued unconditionally -- k-steps are
    // clamped to the last one -- so that the number of loads in flight is the same on every path and the compiler's
    // waits name exactly the load they need)
    load_x(c0 + CH);
    const u32x4* xb = xs + (size_t)stage * XT * 64 + lane;
    u32x4 bq[2][NXP * 4];                                       // the k-step being multiplied and the one after it
#pragma unroll
    for (int i = 0; i < NXP * 4; ++i) bq[0][i] = xb[(size_t)(i * CH) * 64];
#pragma unroll
    for (int u = 0; u < CH; ++u) {
      if (u + 1 < CH) {
#pragma unroll
        for (int i = 0; i < NXP * 4; ++i) bq[(u + 1) & 1][i] = xb[(size_t)(i * CH + u + 1) * 64];
      }
#pragma unroll
      for (int i = 0; i < NXP * 4; ++i) {
        const int t = i & 3;
        acc[0][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, ar[u][0]), __builtin_bit_cast(bf16x8, bq[u & 1][i]), acc[0][t], 0, 0, 0);
        acc[1][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, ar[u][1]), __builtin_bit_cast(bf16x8, bq[u & 1][i]), acc[1][t], 0, 0, 0);
      }
      // use a slot, refill that slot: the weight tiles of the same k-step of the NEXT stage
      const size_t ko = (size_t)min(c0 + CH + u, klast) * 64;
      ar[u][0] = wA[ko]; ar[u][1] = wB[ko];
      __builtin_amdgcn_sched_barrier(0);
    }
    store_x(stage ^ 1);                                         // the other stage was last read before the previous barrier
    // A bare s_barrier behind a wait for this wave's LDS writes only: __syncthreads() carries a work-group fence, for
    // which the compiler drains EVERY outstanding load -- the weight refills issued a moment ago included -- once per
    // stage, which halves the MFMA rate.  All LDS reads of this stage were consumed by the MFMAs above.
    __builtin_amdgcn_s_waitcnt(0xC07F);                         // lgkmcnt(0); vmcnt and expcnt left alone
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
  }
  // accumulator register r of lane l: weight row 8*(r/4) + 4*(l/32) + r%4, activation row l%32; PT[s][m][n], n fastest
  if constexpr (SWIGLU) {
    const int hh = lane >> 5;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      if (!(j ? liveB : liveA)) continue;
      const int rb = j ? rbB : rbA;
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        const int mt = mq * 4 + t;
        if (mt >= MT) continue;
        const int m = mt * 32 + (lane & 31);
        float v[8];                                             // features 4hh + {0..3} and 8 + 4hh + {0..3} of the block
#pragma unroll
        for (int r = 0; r < 8; ++r) {
          const float gs = acc[j][t][r], us = acc[j][t][r + 8];
          v[r] = m < M ? gs / (1.0f + __expf(-gs)) * us : 0.f;
        }
        float x[8];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const float got = __shfl_xor(hh ? v[i] : v[4 + i], 32, 64);   // the partner's features 4..7 (for hh = 0) or 8..11 (for hh = 1)
          x[i] = hh ? got : v[i];
          x[4 + i] = hh ? v[4 + i] : got;
        }
        xf_store8(act, m, 16 * rb + 8 * hh, MT, NRB, NXP, x);
      }
    }
    return;
  }
  const int Mpad = MT * 32;
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    if (!(j ? liveB : liveA)) continue;
    const int rb = j ? rbB : rbA;
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const int mt = mq * 4 + t;
      if (mt >= MT) continue;
      float* out = PT + ((size_t)s * Mpad + mt * 32 + (lane & 31)) * Npad + (size_t)rb * 32 + 4 * (lane >> 5);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        f32x4 v; v.x = acc[j][t][4 * i]; v.y = acc[j][t][4 * i + 1]; v.z = acc[j][t][4 * i + 2]; v.w = acc[j][t][4 * i + 3];
        *(f32x4*)(out + 8 * i) = v;
      }
    }
  }
}

// ============================================================================ row producers
// h[r][:] = embedding of row r's token (fp32).  EmbT = float or bf16_t.
template <typename EmbT>
__global__ __launch_bounds__(256) void k_embed(Pass pass, const TreeDev* tree, SeqState st, const int* tree_tok,
                                               const EmbT* __restrict__ embed, float* __restrict__ h, int d, int vocab) {
  int r = blockIdx.x;
  RowInfo ri = row_info(pass, tree, st, r);
  int tok = 0;
  if (ri.valid) {
    if (pass.kind == PASS_VERIFY) tok = tree_tok[ri.seq * tree->M + ri.node];
    else tok = st.tokens[(size_t)ri.seq * st.tok_stride + ri.pos];
  }
  tok = min(max(tok, 0), vocab - 1);
  for (int k = threadIdx.x; k < d; k += blockDim.x) {
    float v;
    if constexpr (sizeof(EmbT) == 4) v = ((const float*)embed)[(size_t)tok * d + k];
    else v = bf16_to_f32(((const bf16_t*)embed)[(size_t)tok * d + k]);
    h[(size_t)r * d + k] = ri.valid ? v : 0.f;
  }
}

__device__ inline void xf_store8(bf16_t* XF, int m, int k8, int MT, int KS, int nplanes, const float* x) {
  // plane q holds bf16(x - planes 0..q-1), as split_bf16 defines it; written plane by plane so that nothing is indexed
  // by a run-time value (an array indexed by the plane number would live on the stack)
  float r[8];
#pragma unroll
  for (int t = 0; t < 8; ++t) r[t] = x[t];
#pragma unroll
  for (int q = 0; q < 3; ++q) {
    if (q < nplanes) {
      uint32_t b[8];
#pragma unroll
      for (int t = 0; t < 8; ++t) {
        const bf16_t h = f32_to_bf16(r[t]);
        b[t] = h;
        r[t] -= bf16_to_f32(h);
      }
      u32x4 v;
      v.x = b[0] | (b[1] << 16); v.y = b[2] | (b[3] << 16); v.z = b[4] | (b[5] << 16); v.w = b[6] | (b[7] << 16);
      *(u32x4*)(XF + xf_index(m, k8, q, MT, KS)) = v;
    }
  }
}

// Input of the head's FC layer: concat(feature, embedding of the token one step ahead)  (Sec. 3.1).
//   pending pass : feature = target feature kept at the last commit, token = committed token at pos+1
//   level pass   : feature = the head's output at the node's parent, token = the node's drafted token
//   draft prefill: feature = target feature of the prompt position, token = the next prompt token
template <typename EmbT>
__global__ __launch_bounds__(256) void k_fc_input(Pass pass, const TreeDev* tree, SeqState st, const int* tree_tok,
                                                  const float* pend_f /*[seq][D+1][d]*/, const float* node_f /*[seq][M][d]*/,
                                                  const float* chunk_f /*[chunk][d]*/, const EmbT* __restrict__ embed,
                                                  bf16_t* XF, int d, int vocab, int MT, int nplanes) {
  int r = blockIdx.x;
  RowInfo ri = row_info(pass, tree, st, r);
  const int KS = 2 * d / 16;
  const float* f = nullptr;
  int tok = 0;
  if (ri.valid) {
    if (pass.kind == PASS_DRAFT_PENDING) {
      f = pend_f + ((size_t)ri.seq * (tree->D + 1) + ri.rel) * d;
      tok = st.tokens[(size_t)ri.seq * st.tok_stride + ri.pos + 1];
    } else if (pass.kind == PASS_DRAFT_LEVEL) {
      f = node_f + ((size_t)ri.seq * tree->M + tree->parent[ri.node]) * d;
      tok = tree_tok[ri.seq * tree->M + ri.node];
    } else {
      f = chunk_f + (size_t)ri.rel * d;
      tok = st.tokens[(size_t)ri.seq * st.tok_stride + ri.pos + 1];
    }
  }
  tok = min(max(tok, 0), vocab - 1);
  // blockIdx.y splits the 2d columns so that a pass of a few rows still spreads over many CUs
  for (int k8 = (blockIdx.y * blockDim.x + threadIdx.x) * 8; k8 < 2 * d; k8 += gridDim.y * blockDim.x * 8) {
    float x[8];
    for (int t = 0; t < 8; ++t) {
      int k = k8 + t;
      float v = 0.f;
      if (ri.valid) {
        if (k < d) v = f[k];
        else if constexpr (sizeof(EmbT) == 4) v = ((const float*)embed)[(size_t)tok * d + (k - d)];
        else v = bf16_to_f32(((const bf16_t*)embed)[(size_t)tok * d + (k - d)]);
      }
      x[t] = v;
    }
    xf_store8(XF, r, k8, MT, KS, nplanes, x);
  }
}

// h_out[r] = h_in[r] + sum_s PT[s][:, r] + bias ;  x = gain ? rmsnorm(h_out[r]) * gain : h_out[r]
// x goes out in XF layout (GEMM input) and, optionally, as fp32 rows (features).  One block per row.
__global__ __launch_bounds__(256) void k_resnorm(const float* h_in, const float* __restrict__ PT, int S, int Npad, int Mpad,
                                                 const float* bias, float* h_out, const float* gain, float eps,
                                                 bf16_t* XF, int MT, int nplanes, float* xout, int d, const float* row_w) {
  __shared__ float sh[16];
  int r = blockIdx.x;
  float ss = 0.f;
  // each thread owns chunks of 8 consecutive k; the first four chunks (rows of up to 8192 columns) stay in registers
  // for the second phase, further ones are read back from h_out
  constexpr int KEEP = 4;
  float keep[KEEP][8];
  const float rw = row_w ? row_w[r] : 1.0f;    // MoE: this expert's routing weight for the row (0 = not routed here)
  auto phase1 = [&](int k8, float* v) {
    float a[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    if (PT) {
      for (int s0 = 0; s0 < S; s0 += 8) {        // eight splits' worth of loads in flight, added in split order
        f32x4 lo[8], hi[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const float* src = PT + ((size_t)min(s0 + u, S - 1) * Mpad + r) * Npad + k8;
          lo[u] = *(const f32x4*)src; hi[u] = *(const f32x4*)(src + 4);
        }
#pragma unroll
        for (int u = 0; u < 8; ++u)
          if (s0 + u < S) {
            a[0] += lo[u].x; a[1] += lo[u].y; a[2] += lo[u].z; a[3] += lo[u].w;
            a[4] += hi[u].x; a[5] += hi[u].y; a[6] += hi[u].z; a[7] += hi[u].w;
          }
      }
    }
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      int k = k8 + t;
      float x = h_in ? h_in[(size_t)r * d + k] : 0.f;
      if (PT) x += row_w ? rw * a[t] : a[t];
      if (bias) x += bias[k];
      h_out[(size_t)r * d + k] = x;
      ss += x * x;
      v[t] = x;
    }
  };
#pragma unroll
  for (int it = 0; it < KEEP; ++it) {
    const int k8 = (it * (int)blockDim.x + (int)threadIdx.x) * 8;
    if (k8 < d) phase1(k8, keep[it]);
  }
  for (int k8 = (KEEP * blockDim.x + threadIdx.x) * 8; k8 < d; k8 += blockDim.x * 8) { float v[8]; phase1(k8, v); }
  ss = block_sum(ss, sh);
  float rstd = gain ? 1.0f / sqrtf(ss / (float)d + eps) : 1.0f;
  const int KS = d / 16;
  auto phase2 = [&](int k8, const float* v) {
    float x[8];
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      x[t] = gain ? v[t] * rstd * gain[k8 + t] : v[t];
      if (xout) xout[(size_t)r * d + k8 + t] = x[t];
    }
    if (XF) xf_store8(XF, r, k8, MT, KS, nplanes, x);
  };
  if (!XF && !xout) return;
#pragma unroll
  for (int it = 0; it < KEEP; ++it) {
    const int k8 = (it * (int)blockDim.x + (int)threadIdx.x) * 8;
    if (k8 < d) phase2(k8, keep[it]);
  }
  for (int k8 = (KEEP * blockDim.x + threadIdx.x) * 8; k8 < d; k8 += blockDim.x * 8) {
    float v[8];
#pragma unroll
    for (int t = 0; t < 8; ++t) v[t] = h_out[(size_t)r * d + k8 + t];
    phase2(k8, v);
  }
}

// q, k, v = rows of PT (the fused QKV projection); rotate-half RoPE on q and k with the row's position id;
// q -> Q[r][head][dh] fp32, k and v -> this layer's paged cache at the row's slot.
template <typename CT>
__global__ __launch_bounds__(256) void k_qkv_rope_store(Pass pass, const TreeDev* tree, SeqState st,
                                                        const float* __restrict__ PT, int S, int Npad, int Mpad,
                                                        const float* __restrict__ rope_cos, const float* __restrict__ rope_sin,
                                                        float* Q, KVCache kv, int H) {
  // a wave per (row, head); four heads per block
  const int r = blockIdx.x, hd = blockIdx.y * 4 + (threadIdx.x >> 6);
  const int dh = kv.head_dim, half = dh >> 1, KVH = kv.n_kv_heads;
  if (hd >= H + 2 * KVH) return;
  RowInfo ri = row_info(pass, tree, st, r);
  for (int i = threadIdx.x & 63; i < half; i += 64) {
    // q/k heads are packed with rotate-half partners adjacent (PACK_ROPE); v heads keep their order
    int n1 = hd < H + KVH ? hd * dh + 2 * i : hd * dh + i;
    int n2 = hd < H + KVH ? n1 + 1 : n1 + half;
    float a = 0.f, b = 0.f;
    for (int s = 0; s < S; ++s) {
      a += PT[((size_t)s * Mpad + r) * Npad + n1];
      b += PT[((size_t)s * Mpad + r) * Npad + n2];
    }
    if (hd < H + KVH) {   // q or k head: rotate
      float c = rope_cos[(size_t)ri.pos * half + i], sn = rope_sin[(size_t)ri.pos * half + i];
      float a2 = a * c - b * sn, b2 = b * c + a * sn;
      a = a2; b = b2;
    }
    if (hd < H) {
      Q[((size_t)r * H + hd) * dh + i] = a;
      Q[((size_t)r * H + hd) * dh + i + half] = b;
    } else if (ri.valid) {
      int kvh = (hd - H) % KVH;
      CT* base = (CT*)(hd < H + KVH ? kv.k : kv.v) + kv_offset(kv, ri.seq, ri.slot, kvh);
      cache_store(base + i, a);
      cache_store(base + i + half, b);
    }
  }
}

// (Tree-masked paged attention for both paths is k2_attn, in kernels2.h.)

// ============================================================================ SwiGLU and logits epilogues
// act[r][k] = silu(gate) * up with the fused matrix's row order (PACK_GATE / PACK_UP)   (F = d_ffn)
// A wave owns one tile of the output (32 rows x one k-step of 16 features): lane = (row, half of the k-step), which is
// the tile's own lane order, so the wave writes 1 KiB contiguous per plane; the lane's 8 gate and 8 up values are
// 32 bytes each in the row's 128-byte line of the fused block, so the two lanes of a row read that line exactly once.
// Grid (k-steps / 4, 32-row tiles); rows beyond M are written as zeros.
__global__ __launch_bounds__(256) void k_swiglu(const float* __restrict__ PT, int S, int Npad, int Mpad, int F, int M,
                                                bf16_t* XF, int MT, int nplanes) {
  const int lane = threadIdx.x & 63, ks = blockIdx.x * 4 + (threadIdx.x >> 6), KSF = F / 16;
  if (ks >= KSF) return;
  const int r = blockIdx.y * 32 + (lane & 31), half = lane >> 5;
  const int ng = 32 * ks + 8 * half;                 // this lane's 8 gate rows of the fused matrix; the up rows sit 16 further
  float gs[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f}, us[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  if (r < M) {
    for (int s0 = 0; s0 < S; s0 += 4) {              // four splits' worth of loads in flight, added in split order
      f32x4 g0[4], g1[4], u0[4], u1[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const float* src = PT + ((size_t)min(s0 + q, S - 1) * Mpad + r) * Npad + ng;
        g0[q] = *(const f32x4*)src; g1[q] = *(const f32x4*)(src + 4);
        u0[q] = *(const f32x4*)(src + 16); u1[q] = *(const f32x4*)(src + 20);
      }
#pragma unroll
      for (int q = 0; q < 4; ++q)
        if (s0 + q < S) {
          gs[0] += g0[q].x; gs[1] += g0[q].y; gs[2] += g0[q].z; gs[3] += g0[q].w;
          gs[4] += g1[q].x; gs[5] += g1[q].y; gs[6] += g1[q].z; gs[7] += g1[q].w;
          us[0] += u0[q].x; us[1] += u0[q].y; us[2] += u0[q].z; us[3] += u0[q].w;
          us[4] += u1[q].x; us[5] += u1[q].y; us[6] += u1[q].z; us[7] += u1[q].w;
        }
    }
  }
  float x[8];
#pragma unroll
  for (int t = 0; t < 8; ++t) x[t] = r < M ? gs[t] / (1.0f + __expf(-gs[t])) * us[t] : 0.f;
  xf_store8(XF, r, 16 * ks + 8 * half, MT, KSF, nplanes, x);
}

// logits[dst_row(r)][v] = sum_s PT[s][v][r].  Where a pass's row maps to no output (padding rows, pending rows
// other than the root pair) nothing is written.  out_kind 0: per-node buffer [seq][M][V]; 1: per-seq [seq][V].
__global__ __launch_bounds__(256) void k_logits(Pass pass, const TreeDev* tree, SeqState st, const float* __restrict__ PT,
                                                int S, int Npad, int Mpad, float* out, int out_kind, int V, int only_last_row) {
  int r = blockIdx.y;
  RowInfo ri = row_info(pass, tree, st, r);
  if (!ri.valid) return;
  size_t dst;
  if (out_kind == 0) {
    if (ri.node < 0) return;
    dst = ((size_t)ri.seq * tree->M + ri.node) * V;
  } else {
    if (only_last_row && ri.rel != pass.chunk_n - 1 && pass.kind != PASS_VANILLA) return;
    dst = (size_t)ri.seq * V;
  }
  int v = blockIdx.x * blockDim.x + threadIdx.x;
  if (v >= V) return;
  float a = 0.f;
  for (int s = 0; s < S; ++s) a += PT[((size_t)s * Mpad + r) * Npad + v];
  out[dst + v] = a;
}

// copy rows (features): dst[dst_row(r)] = src[r]
__global__ __launch_bounds__(256) void k_store_rows(Pass pass, const TreeDev* tree, SeqState st, const float* src,
                                                    float* node_dst /*[seq][M][d]*/, float* pend_dst /*[seq][D+1][d]*/,
                                                    float* chunk_dst /*[chunk][d]*/, int d) {
  int r = blockIdx.x;
  RowInfo ri = row_info(pass, tree, st, r);
  if (!ri.valid) return;
  float* dst = nullptr;
  if (pass.kind == PASS_VERIFY || pass.kind == PASS_DRAFT_LEVEL) dst = node_dst + ((size_t)ri.seq * tree->M + ri.node) * d;
  else if (pass.kind == PASS_DRAFT_PENDING) { if (ri.node == 0) dst = node_dst + ((size_t)ri.seq * tree->M) * d; }
  else if (pass.kind == PASS_PREFILL_T) {
    dst = chunk_dst + (size_t)ri.rel * d;
  } else if (pass.kind == PASS_VANILLA) dst = pend_dst + (size_t)ri.seq * (tree->D + 1) * d;
  if (!dst) return;
  for (int k = threadIdx.x; k < d; k += blockDim.x) dst[k] = src[(size_t)r * d + k];
}

// ============================================================================ training loss of the head (Sec. 3.2)
// Rows of fp32 features -> rows [row0, row0 + rows) of a GEMM input of MT 32-row tiles (XF layout).  Grid (rows, parts).
__global__ __launch_bounds__(256) void k_rows_to_xf(const float* __restrict__ src, int row0, bf16_t* XF, int MT, int nplanes, int d) {
  const int r = blockIdx.x;
  for (int k8 = (blockIdx.y * blockDim.x + threadIdx.x) * 8; k8 < d; k8 += gridDim.y * blockDim.x * 8) {
    float x[8];
    const f32x4 a = *(const f32x4*)(src + (size_t)r * d + k8), b = *(const f32x4*)(src + (size_t)r * d + k8 + 4);
    x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w; x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
    xf_store8(XF, row0 + r, k8, MT, d / 16, nplanes, x);
  }
}

// One row of the loss (block = row r of the pass).  Z holds the LM head's logits of the pass as S split-K partials
// PT[s][m][n]: row r = logits of the label feature f, row zh_row0 + r = logits of the prediction fhat.
//   p = softmax(z), q = softmax(zh);  cross entropy of the row = lse(zh) - sum_v p_v zh_v
//   dZ[r][v] = (q_v - p_v) * cls_scale            (cls_scale = w_cls / rows of the whole call), written as GEMM input
//   Smooth L1 of the row over d columns (threshold 1), its derivative clip(x, -1, 1) * reg_scale -> grad[r][:]
// row_loss[r] = (sum of the row's smooth-L1 terms, the row's cross entropy); means are taken by the caller.
// NCH > 0: a thread keeps its NCH chunks of 8 logits of both rows in registers (V <= 8192 * NCH), so the logits are
// read once; NCH = 0: any V, three passes over the logits.
template <int NCH>
__global__ __launch_bounds__(1024) void k_head_loss_row(const float* __restrict__ Z, int S, int Mpad, int Npad, int zh_row0, int V,
                                                        const float* __restrict__ f, const float* __restrict__ fhat, int d,
                                                        float cls_scale, float reg_scale, bf16_t* DZ, int MT, int nplanes,
                                                        float* grad /*[rows][d] or null*/, float* row_loss /*[rows][2]*/) {
  __shared__ float sh[16];
  const int r = blockIdx.x;
  auto load8 = [&](int row, int v8, float* x) {
    f32x4 a = {0.f, 0.f, 0.f, 0.f}, b = {0.f, 0.f, 0.f, 0.f};
    for (int s = 0; s < S; ++s) {
      const float* src = Z + ((size_t)s * Mpad + row) * Npad + v8;
      const f32x4 a1 = *(const f32x4*)src, b1 = *(const f32x4*)(src + 4);
      a += a1; b += b1;
    }
    x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w; x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
  };
  constexpr int NR = NCH > 0 ? NCH : 1;
  float zr[NR][8], hr[NR][8];
  float mz = -INFINITY, mh = -INFINITY;
  if constexpr (NCH > 0) {
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
      const int v8 = (c * 1024 + (int)threadIdx.x) * 8;
      if (v8 < V) {
        load8(r, v8, zr[c]); load8(zh_row0 + r, v8, hr[c]);
#pragma unroll
        for (int t = 0; t < 8; ++t) { mz = fmaxf(mz, zr[c][t]); mh = fmaxf(mh, hr[c][t]); }
      }
    }
  } else {
    for (int v8 = threadIdx.x * 8; v8 < V; v8 += blockDim.x * 8) {
      load8(r, v8, zr[0]); load8(zh_row0 + r, v8, hr[0]);
#pragma unroll
      for (int t = 0; t < 8; ++t) { mz = fmaxf(mz, zr[0][t]); mh = fmaxf(mh, hr[0][t]); }
    }
  }
  mz = block_max(mz, sh);
  mh = block_max(mh, sh);
  float sz = 0.f, shh = 0.f, dot = 0.f;
  auto sums8 = [&](const float* z, const float* zh) {
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      const float e = __expf(z[t] - mz);
      sz += e; shh += __expf(zh[t] - mh); dot += e * (zh[t] - mh);
    }
  };
  if constexpr (NCH > 0) {
#pragma unroll
    for (int c = 0; c < NCH; ++c)
      if ((c * 1024 + (int)threadIdx.x) * 8 < V) sums8(zr[c], hr[c]);
  } else {
    for (int v8 = threadIdx.x * 8; v8 < V; v8 += blockDim.x * 8) { load8(r, v8, zr[0]); load8(zh_row0 + r, v8, hr[0]); sums8(zr[0], hr[0]); }
  }
  sz = block_sum(sz, sh);
  shh = block_sum(shh, sh);
  dot = block_sum(dot, sh);
  const float cls = logf(shh) - dot / sz;                          // lse(zh) - sum_v p_v zh_v, both taken relative to mh
  const float isz = 1.0f / sz, ish = 1.0f / shh;
  auto store8 = [&](int v8, const float* z, const float* zh) {
    float x[8];
#pragma unroll
    for (int t = 0; t < 8; ++t) x[t] = (__expf(zh[t] - mh) * ish - __expf(z[t] - mz) * isz) * cls_scale;
    xf_store8(DZ, r, v8, MT, V / 16, nplanes, x);
  };
  if constexpr (NCH > 0) {
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
      const int v8 = (c * 1024 + (int)threadIdx.x) * 8;
      if (v8 < V) store8(v8, zr[c], hr[c]);
    }
  } else {
    for (int v8 = threadIdx.x * 8; v8 < V; v8 += blockDim.x * 8) { load8(r, v8, zr[0]); load8(zh_row0 + r, v8, hr[0]); store8(v8, zr[0], hr[0]); }
  }
  float reg = 0.f;
  for (int k = threadIdx.x; k < d; k += blockDim.x) {
    const float x = fhat[(size_t)r * d + k] - f[(size_t)r * d + k];
    const float ax = fabsf(x);
    reg += ax < 1.0f ? 0.5f * x * x : ax - 0.5f;
    if (grad) grad[(size_t)r * d + k] = fminf(fmaxf(x, -1.0f), 1.0f) * reg_scale;
  }
  reg = block_sum(reg, sh);
  if (threadIdx.x == 0) { row_loss[2 * r] = reg; row_loss[2 * r + 1] = cls; }
}

// grad[r][k] += sum over the S split-K partials of (dZ W)[r][k]   (the classification part of the gradient)
__global__ __launch_bounds__(256) void k_head_loss_grad_finish(const float* __restrict__ PT, int S, int Mpad, int Npad, float* grad, int d) {
  const int r = blockIdx.y, k = blockIdx.x * blockDim.x + threadIdx.x;
  if (k >= d) return;
  float a = 0.f;
  for (int s = 0; s < S; ++s) a += PT[((size_t)s * Mpad + r) * Npad + k];
  grad[(size_t)r * d + k] += a;
}

// acc[0] += sum of the rows' smooth-L1 sums, acc[1] += sum of the rows' cross entropies, in fp64 and in a fixed order:
// lane l of one wave adds rows l, l + 64, ...; lane 0 then adds the 64 lane sums in lane order.
__global__ __launch_bounds__(64) void k_head_loss_accumulate(const float* row_loss, int rows, double* acc) {
  __shared__ double sa[64], sb[64];
  double a = 0.0, b = 0.0;
  for (int r = threadIdx.x; r < rows; r += 64) { a += (double)row_loss[2 * r]; b += (double)row_loss[2 * r + 1]; }
  sa[threadIdx.x] = a; sb[threadIdx.x] = b;
  __syncthreads();
  if (threadIdx.x == 0) {
    double ta = acc[0], tb = acc[1];
    for (int l = 0; l < 64; ++l) { ta += sa[l]; tb += sb[l]; }
    acc[0] = ta; acc[1] = tb;
  }
}

// out = in + amplitude * n, n = the odd multiple of 2^-24 in (-1, 1) that the counter-based generator draws for
// (row, column); the product and the sum are rounded separately (no fused multiply-add), so the result is the same
// bits wherever it is computed.
__global__ __launch_bounds__(256) void k_feature_noise(const float* in, float* out, int rows, int d, float amplitude, unsigned long long prefix) {
#pragma clang fp contract(off)
  const size_t n = (size_t)rows * d;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) {
    const uint32_t r = (uint32_t)(i / d), k = (uint32_t)(i % d);
    const int k24 = (int)rng_u24(prefix, r >> 16, r & 0xFFFFu, k);
    const float u = (float)(2 * (k24 - (1 << 23)) + 1) * 5.9604644775390625e-8f;
    const float prod = amplitude * u;
    out[i] = in[i] + prod;
  }
}

// ============================================================================ token choice
struct HintDev {
  const int* future;     // [max_batch][stride]
  int stride;
  const int* n;          // [max_batch] tokens known (0 = off)
  const float* alpha;    // [max_batch]
  const float* bias;
  const unsigned long long* seed;
};

// Children of one tree node = the top-k entries of its (knob-adjusted, Gumbel-perturbed when non-greedy) head
// logits, rank r = (r+1)-th largest, equal scores -> lower token id (App. A.1).  Block = (parent row, seq).
template <bool BIGV>   // BIGV: more than 32768 vocabulary entries (the scores of a row do not fit the block's registers)
__global__ __launch_bounds__(1024) void k_expand(int level /*-1 = root*/, int n_seq, const TreeDev* tree, SeqState st,
                                                 float* draft_logits /*[seq][M][V]*/, int* tree_tok, int* on_path, HintDev hint,
                                                 int V, float temperature, unsigned long long rng_seed, unsigned long long* trace,
                                                 const float* __restrict__ feat_src /*[pass rows][d] or null*/, float* node_f /*[seq][M][d]*/,
                                                 int d, int src_rows_per_seq) {
  __shared__ float shv[16];
  __shared__ int shi[16];
  const int seq = blockIdx.y;
  unsigned long long* tr = TRACE_PTR((trace && threadIdx.x == 0 && blockIdx.x == 0 && seq == 0) ? trace : nullptr);
  TRACE_STAMP(tr, 0);
  const int v = level < 0 ? 0 : tree->level_rows[level][blockIdx.x];
  const int M = tree->M;
  // The node's own head feature (the row of the pass that produced these logits) goes to node_f here when the caller
  // asks for it: one block per row of the pass exists anyway, which saves a separate copy kernel per pass.
  // Row of the pass: a level pass lists the level's parent nodes in order; in a pending pass the root is the
  // sequence's last pending row.
  if (feat_src) {
    const int row = seq * src_rows_per_seq + (level < 0 ? max(st.n_pend[seq] - 1, 0) : (int)blockIdx.x);
    const float* src = feat_src + (size_t)row * d;
    float* dst = node_f + ((size_t)seq * M + v) * d;
    for (int k = threadIdx.x; k < d; k += blockDim.x) dst[k] = src[k];
  }
  float* lg = draft_logits + ((size_t)seq * M + v) * V;
  // Loads are grouped by what they depend on, so that the kernel pays two memory round trips, not one per fact:
  // (1) everything addressed by (seq, v) alone, including the first 32 logits of every thread ...
  constexpr int XPT = 32;                                      // logits per thread and chunk (1024 threads: 32768)
  float x[XPT];
#pragma unroll
  for (int u = 0; u < XPT; ++u) x[u] = lg[min(u * 1024 + (int)threadIdx.x, V - 1)];
  const int n = st.n_tok[seq];
  const int hn = hint.n[seq];
  const unsigned long long hseed = hint.seed[seq];
  const float halpha = hint.alpha[seq], hbias = hint.bias[seq];
  const int depth_v = tree->depth[v], nk = tree->nchild[v];
  const int on_v = v == 0 ? 0 : on_path[seq * M + v];
  const unsigned long long step_no = (unsigned long long)st.step_no[seq];
  // (2) ... then what needs the sequence length: the root token, the target's future tokens at two positions
  const int stride = hint.stride;
  const int pos_child = n + depth_v;
  const int root_tok = st.tokens[(size_t)seq * st.tok_stride + max(n - 1, 0)];
  const int fut_root = hint.future[(size_t)seq * stride + min(max(n - 1, 0), stride - 1)];
  const int fut_child = hint.future[(size_t)seq * stride + min(pos_child, stride - 1)];
  int on = on_v;
  if (v == 0) {
    on = (hn > n - 1) && fut_root == root_tok;
    if (threadIdx.x == 0) { tree_tok[seq * M] = root_tok; on_path[seq * M] = on; }
  }
  // acceptance knob of the synthetic workload
  const int hinted = (on && pos_child < hn) ? fut_child : -1;
  float adj = 0.f;
  if (hinted >= 0) {
    uint32_t k24 = rng_u24(rng_prefix(hseed, PURPOSE_HINT, 0), (uint32_t)seq, 0, (uint32_t)pos_child);
    adj = ((float)k24 * 5.9604644775390625e-8f < halpha) ? hbias : -hbias;
  }
  const bool gumbel = temperature > 0.f;
  unsigned long long pre = 0ull;
  if (gumbel) pre = rng_prefix(rng_seed, PURPOSE_GUMBEL, step_no);
  int childs[EAGLE_MAX_CHILD];
#pragma unroll
  for (int q = 0; q < EAGLE_MAX_CHILD; ++q) childs[q] = tree->child[v][q];
  int picked[EAGLE_MAX_CHILD];                                 // thread 0 writes the results once, after the rounds
#pragma unroll
  for (int q = 0; q < EAGLE_MAX_CHILD; ++q) picked[q] = 0;
  TRACE_STAMP_AFTER(tr, 1, x[0]);
  if constexpr (!BIGV) {
    // Scores stay in registers.  Every thread offers its best entry; the block picks the overall best (ties to the
    // lower token id); only the thread that owned it removes it and looks for its next best.
#pragma unroll
    for (int u = 0; u < XPT; ++u) {
      const int j = u * 1024 + (int)threadIdx.x;
      float sc = x[u];
      if (j == hinted) { sc += adj; lg[j] = sc; }            // later phases read the adjusted logits
      if (gumbel) {
        float un = ((float)rng_u24(pre, (uint32_t)seq, (uint32_t)v, (uint32_t)min(j, V - 1)) + 0.5f) * 5.9604644775390625e-8f;
        sc = sc / temperature - logf(-logf(un));
      }
      x[u] = j < V ? sc : -INFINITY;
    }
    float lv = -INFINITY; int li = 0x7fffffff;
#pragma unroll
    for (int u = 0; u < XPT; ++u) better(lv, li, x[u], u * 1024 + (int)threadIdx.x);
    TRACE_STAMP_AFTER(tr, 2, lv);
    for (int r = 0; r < nk; ++r) {
      float bv = lv; int bi = li;
      block_argmax(bv, bi, shv, shi);
      if (bi == li) {                                           // mine: take it out, find my next best
        lv = -INFINITY; li = 0x7fffffff;
#pragma unroll
        for (int u = 0; u < XPT; ++u) {
          const int j = u * 1024 + (int)threadIdx.x;
          if (j == bi) x[u] = -INFINITY;
          better(lv, li, x[u], j);
        }
        if (lv == -INFINITY) li = 0x7fffffff;
      }
#pragma unroll
      for (int q = 0; q < EAGLE_MAX_CHILD; ++q) if (q == r) picked[q] = bi;
      __syncthreads();                                          // shv / shi are reused by the next round
    }
  } else {
    // Larger vocabularies: one pass with a per-thread sorted top-nk list, then rounds over the lists' heads.
    float tv[EAGLE_MAX_CHILD];
    int ti[EAGLE_MAX_CHILD];
#pragma unroll
    for (int q = 0; q < EAGLE_MAX_CHILD; ++q) { tv[q] = -INFINITY; ti[q] = 0x7fffffff; }
    for (int j0 = 0; j0 < V; j0 += XPT * 1024) {
      if (j0 > 0) {
#pragma unroll
        for (int u = 0; u < XPT; ++u) x[u] = lg[min(j0 + u * 1024 + (int)threadIdx.x, V - 1)];
      }
#pragma unroll
      for (int u = 0; u < XPT; ++u) {
        const int j = j0 + u * 1024 + (int)threadIdx.x;
        if (j >= V) continue;
        float sc = x[u];
        if (j == hinted) { sc += adj; lg[j] = sc; }
        if (gumbel) {
          float un = ((float)rng_u24(pre, (uint32_t)seq, (uint32_t)v, (uint32_t)j) + 0.5f) * 5.9604644775390625e-8f;
          sc = sc / temperature - logf(-logf(un));
        }
        float cv = sc; int ci = j;
#pragma unroll
        for (int q = 0; q < EAGLE_MAX_CHILD; ++q) {
          const bool win = cv > tv[q] || (cv == tv[q] && ci < ti[q]);
          const float ov = tv[q]; const int oi = ti[q];
          if (win) { tv[q] = cv; ti[q] = ci; cv = ov; ci = oi; }
        }
      }
    }
    for (int r = 0; r < nk; ++r) {
      float bv = tv[0]; int bi = ti[0];
      block_argmax(bv, bi, shv, shi);
      if (bi == ti[0]) {
#pragma unroll
        for (int q = 0; q + 1 < EAGLE_MAX_CHILD; ++q) { tv[q] = tv[q + 1]; ti[q] = ti[q + 1]; }
        tv[EAGLE_MAX_CHILD - 1] = -INFINITY; ti[EAGLE_MAX_CHILD - 1] = 0x7fffffff;
      }
#pragma unroll
      for (int q = 0; q < EAGLE_MAX_CHILD; ++q) if (q == r) picked[q] = bi;
      __syncthreads();
    }
  }
  if (threadIdx.x == 0) {
#pragma unroll
    for (int q = 0; q < EAGLE_MAX_CHILD; ++q)
      if (q < nk) {
        tree_tok[seq * M + childs[q]] = picked[q];
        on_path[seq * M + childs[q]] = (hinted >= 0 && picked[q] == hinted);
      }
  }
  TRACE_STAMP(tr, 3);
}

// softmax(x / T) over V entries into p (block-wide), returns nothing; sh >= 16 floats
__device__ inline void block_softmax(const float* x, float* p, int V, float invT, float* sh) {
  float mx = -INFINITY;
  for (int j = threadIdx.x; j < V; j += blockDim.x) mx = fmaxf(mx, x[j] * invT);
  mx = block_max(mx, sh);
  float sm = 0.f;
  for (int j = threadIdx.x; j < V; j += blockDim.x) { float e = expf(x[j] * invT - mx); p[j] = e; sm += e; }
  sm = block_sum(sm, sh);
  for (int j = threadIdx.x; j < V; j += blockDim.x) p[j] = p[j] / sm;
  __syncthreads();
}

// smallest x with cumsum(p)[x] > u * sum(p); block-wide, result broadcast through *res (shared).  The running sum is
// carried in fp64: with 32000 entries a bin is ~3e-5 wide, which an fp32 running sum cannot resolve -- the draw would
// depend on the order of the additions instead of on p.  (Thread chunks, then a prefix over the chunk sums, then a
// sequential walk of the one chunk that holds the target: fixed order.)
__device__ inline int block_inverse_cdf(const float* p, int V, float u, double* sh_d /*>= blockDim.x + 1*/, int* res) {
  const int nt = blockDim.x;
  const int per = (V + nt - 1) / nt;
  const int j0 = threadIdx.x * per, j1 = min(V, j0 + per);
  double s = 0.0;
  for (int j = j0; j < j1; ++j) s += (double)p[j];
  sh_d[threadIdx.x] = s;
  __syncthreads();
  if (threadIdx.x == 0) {
    double tot = 0.0;
    for (int i = 0; i < nt; ++i) { double t = sh_d[i]; sh_d[i] = tot; tot += t; }   // exclusive prefix, fixed order
    sh_d[nt] = tot;
    *res = V - 1;
  }
  __syncthreads();
  const double target = (double)u * sh_d[nt];
  double c = sh_d[threadIdx.x];
  const double nxt = threadIdx.x + 1 < nt ? sh_d[threadIdx.x + 1] : sh_d[nt];
  __syncthreads();
  if (j0 < j1 && c <= target && (target < nxt || threadIdx.x + 1 == nt || j1 == V)) {
    int found = -1, last_pos = -1;
    for (int j = j0; j < j1; ++j) {
      if (p[j] > 0.f) last_pos = j;
      c += (double)p[j];
      if (c > target) { found = j; break; }
    }
    if (found < 0) found = last_pos;            // rounding left the running sum just short of the target
    if (found >= 0) atomicMin(res, found);
  }
  __syncthreads();
  return *res;
}

// Pick the next token of every sequence from logits[seq][V] (prefill's first token, vanilla decoding):
// argmax when greedy, else one inverse-CDF draw from softmax(logits / T).  Also advances the sequence state.
__global__ __launch_bounds__(1024) void k_choose(SeqState st, int seq0, const float* logits, int V, float temperature,
                                                 unsigned long long rng_seed, float* pbuf /*[seq][V]*/, int is_prefill,
                                                 int prefill_n, int max_pend) {
  __shared__ float shv[16];
  __shared__ int shi[16];
  __shared__ double sh_f[1025];
  __shared__ int res;
  const int seq = seq0 + blockIdx.x;
  const float* lg = logits + (size_t)seq * V;
  int tok;
  if (temperature <= 0.f) {
    float bv = -INFINITY; int bi = 0x7fffffff;
    for (int j = threadIdx.x; j < V; j += blockDim.x) better(bv, bi, lg[j], j);
    block_argmax(bv, bi, shv, shi);
    tok = bi;
  } else {
    float* p = pbuf + (size_t)seq * V;
    block_softmax(lg, p, V, 1.0f / temperature, shv);
    int step = is_prefill ? 0 : st.step_no[seq];
    float u = (float)rng_u24(rng_prefix(rng_seed, PURPOSE_FINAL, (unsigned long long)step), (uint32_t)seq, 0, 0) * 5.9604644775390625e-8f;
    tok = block_inverse_cdf(p, V, u, sh_f, &res);
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    if (is_prefill) {
      st.tokens[(size_t)seq * st.tok_stride + prefill_n] = tok;
      st.n_tok[seq] = prefill_n + 1; st.ctx_len[seq] = prefill_n; st.n_pend[seq] = 1; st.step_no[seq] = 1;
    } else {
      int n = st.n_tok[seq];
      st.tokens[(size_t)seq * st.tok_stride + n] = tok;
      st.n_tok[seq] = n + 1; st.ctx_len[seq] += 1; st.n_pend[seq] = max_pend + 1 /* head is stale after vanilla */;
      st.step_no[seq] += 1;
    }
  }
}

// Acceptance (Sec. 2; App. A.2, Alg. 1 applied recursively at every node).  Block = one sequence.
//   greedy : follow the child whose token equals argmax of the target logits at the current node
//   T > 0  : children in rank order, accept child i when r * q_i(t_i) < p(t_i); on rejection
//            p <- norm(max(0, p - q_i)) and q_{i+1} = q_i without t_i, renormalised (children were drawn
//            without replacement); when nothing is accepted draw the bonus token from what is left of p.
// arg-max token of every row of logits (lowest id among equals), one block per row: the greedy walk below visits up
// to depth + 1 nodes one after the other, and scanning their rows there would run on a single CU
__global__ __launch_bounds__(1024) void k_row_argmax(const float* __restrict__ L, int V, int* __restrict__ amax) {
  __shared__ float shv[16];
  __shared__ int shi[16];
  const float* lg = L + (size_t)blockIdx.x * V;
  float bv = -INFINITY; int bi = 0x7fffffff;
  for (int j = threadIdx.x; j < V; j += blockDim.x) better(bv, bi, lg[j], j);
  block_argmax(bv, bi, shv, shi);
  if (threadIdx.x == 0) amax[blockIdx.x] = bi;
}

__global__ __launch_bounds__(1024) void k_accept(const TreeDev* tree, SeqState st, const float* L /*[seq][M][V]*/,
                                                 const float* draft_logits, const int* tree_tok, int V, float temperature,
                                                 unsigned long long rng_seed, float* pbuf, float* qbuf,
                                                 int* path_out /*[seq][D+1]*/, int* tok_out, int* len_out,
                                                 const int* __restrict__ amax /*[seq][M], greedy only*/) {
  __shared__ float shv[16];
  __shared__ int shi[16];
  __shared__ double sh_f[1025];
  __shared__ int res, s_next;
  const int seq = blockIdx.x, M = tree->M, D1 = tree->D + 1;
  int cur = 0, len = 1, bonus = 0;
  if (threadIdx.x == 0) path_out[seq * D1] = 0;
  const int step = st.step_no[seq];
  while (true) {
    const float* lg = L + ((size_t)seq * M + cur) * V;
    const int nk = tree->nchild[cur];
    if (temperature <= 0.f) {
      const int bi = amax[seq * M + cur];
      if (threadIdx.x == 0) {
        s_next = -1;
        for (int r = 0; r < nk; ++r) {
          int c = tree->child[cur][r];
          if (tree_tok[seq * M + c] == bi) { s_next = c; break; }
        }
      }
      __syncthreads();
      if (s_next < 0) { bonus = bi; break; }
    } else {
      float* p = pbuf + (size_t)seq * V;
      float* q = qbuf + (size_t)seq * V;
      const float invT = 1.0f / temperature;
      block_softmax(lg, p, V, invT, shv);
      if (nk > 0) block_softmax(draft_logits + ((size_t)seq * M + cur) * V, q, V, invT, shv);
      if (threadIdx.x == 0) s_next = -1;
      __syncthreads();
      for (int r = 0; r < nk; ++r) {
        const int c = tree->child[cur][r];
        const int t = tree_tok[seq * M + c];
        float rr = (float)rng_u24(rng_prefix(rng_seed, PURPOSE_ACCEPT, (unsigned long long)step), (uint32_t)seq, (uint32_t)c, 0) * 5.9604644775390625e-8f;
        bool ok = rr * q[t] < p[t];
        __syncthreads();
        if (ok) { if (threadIdx.x == 0) s_next = c; break; }
        // residual target, proposal without t
        float sm = 0.f;
        for (int j = threadIdx.x; j < V; j += blockDim.x) { float d = fmaxf(p[j] - q[j], 0.f); sm += d; }
        sm = block_sum(sm, shv);
        if (sm > 1e-20f)
          for (int j = threadIdx.x; j < V; j += blockDim.x) p[j] = fmaxf(p[j] - q[j], 0.f) / sm;
        __syncthreads();
        if (threadIdx.x == 0) q[t] = 0.f;
        __syncthreads();
        float qs = 0.f;
        for (int j = threadIdx.x; j < V; j += blockDim.x) qs += q[j];
        qs = block_sum(qs, shv);
        if (qs > 0.f)
          for (int j = threadIdx.x; j < V; j += blockDim.x) q[j] = q[j] / qs;
        __syncthreads();
      }
      __syncthreads();
      if (s_next < 0) {
        float u = (float)rng_u24(rng_prefix(rng_seed, PURPOSE_FINAL, (unsigned long long)step), (uint32_t)seq, (uint32_t)cur, 0) * 5.9604644775390625e-8f;
        bonus = block_inverse_cdf(p, V, u, sh_f, &res);
        break;
      }
    }
    cur = s_next;
    if (threadIdx.x == 0) path_out[seq * D1 + len] = cur;
    ++len;
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    const int n = st.n_tok[seq];
    for (int i = 1; i < len; ++i) {
      int t = tree_tok[seq * M + path_out[seq * D1 + i]];
      tok_out[seq * D1 + i - 1] = t;
      st.tokens[(size_t)seq * st.tok_stride + n + i - 1] = t;
    }
    tok_out[seq * D1 + len - 1] = bonus;
    st.tokens[(size_t)seq * st.tok_stride + n + len - 1] = bonus;
    len_out[seq] = len;
    st.commit_base[seq] = st.ctx_len[seq];
    st.n_tok[seq] = n + len; st.ctx_len[seq] += len; st.n_pend[seq] = len; st.step_no[seq] = step + 1;
  }
}

// Commit (Sec. 3.3: accepted tokens and their features are kept): for every layer, KV rows of the accepted
// nodes move from slot base+path[i] to base+i, and the accepted nodes' target features become the pending
// features of the next drafting phase.  ONE launch: blockIdx.y = layer (last y = the feature rows).
// A thread owns one 16-byte column of a row and moves i = 1..len-1 in increasing order; since path[i] >= i and
// path is increasing, a destination is never a source that is still to be read.
template <typename CT>
__global__ __launch_bounds__(256) void k_compact(const TreeDev* tree, SeqState st, const int* path, const int* len_p,
                                                 void* kcache, void* vcache, size_t layer_stride_elems, int n_layers,
                                                 KVCache kv, const float* F /*[seq][M][d]*/, float* pend_f, int d) {
  const int seq = blockIdx.z, layer = blockIdx.y;
  const int D1 = tree->D + 1, M = tree->M;
  const int len = len_p[seq];
  const int* pth = path + seq * D1;
  if (layer == n_layers) {
    for (int i = 0; i < len; ++i) {
      const float* src = F + ((size_t)seq * M + pth[i]) * d;
      float* dst = pend_f + ((size_t)seq * D1 + i) * d;
      for (int k = blockIdx.x * blockDim.x + threadIdx.x; k < d; k += gridDim.x * blockDim.x) dst[k] = src[k];
    }
    return;
  }
  const int base = st.commit_base[seq];
  constexpr int EPC = 16 / sizeof(CT);                        // elements per 16-byte column
  const int cols = kv.n_kv_heads * kv.head_dim / EPC;
  kv.k = (CT*)kcache + (size_t)layer * layer_stride_elems;
  kv.v = (CT*)vcache + (size_t)layer * layer_stride_elems;
  for (int c = blockIdx.x * blockDim.x + threadIdx.x; c < 2 * cols; c += gridDim.x * blockDim.x) {
    const int which = c / cols, cc = c % cols;
    const int kvh = cc * EPC / kv.head_dim, off = cc * EPC % kv.head_dim;
    CT* cache = (CT*)(which ? kv.v : kv.k);
    for (int i = 1; i < len; ++i) {
      if (pth[i] == i) continue;
      u32x4 val = *(const u32x4*)(cache + kv_offset(kv, seq, base + pth[i], kvh) + off);
      *(u32x4*)(cache + kv_offset(kv, seq, base + i, kvh) + off) = val;
    }
  }
}

// Commit of paths handed in by the caller instead of found by k_accept (lock-step tests drive the engine along the
// oracle's choices with it): the bookkeeping at the end of k_accept, for every sequence.  bonus[seq] = the token that
// follows the accepted drafts.  k_compact runs afterwards as in a normal step.
__global__ void k_force_commit(const TreeDev* tree, SeqState st, const int* path /*[seq][D+1]*/, const int* len_p,
                               const int* bonus, const int* tree_tok, int* tok_out, int n_seq) {
  const int seq = blockIdx.x * blockDim.x + threadIdx.x;
  if (seq >= n_seq) return;
  const int M = tree->M, D1 = tree->D + 1, len = len_p[seq], n = st.n_tok[seq];
  for (int i = 1; i < len; ++i) {
    const int t = tree_tok[seq * M + path[seq * D1 + i]];
    tok_out[seq * D1 + i - 1] = t;
    st.tokens[(size_t)seq * st.tok_stride + n + i - 1] = t;
  }
  tok_out[seq * D1 + len - 1] = bonus[seq];
  st.tokens[(size_t)seq * st.tok_stride + n + len - 1] = bonus[seq];
  st.commit_base[seq] = st.ctx_len[seq];
  st.n_tok[seq] = n + len; st.ctx_len[seq] += len; st.n_pend[seq] = len; st.step_no[seq] += 1;
}

// ============================================================================ MoE router
// Row r: x = the normalised MLP input (given, or h * rstd * gain), router logits in fp32, top-k experts (equal
// logits -> lower expert id), softmax over the selected logits.  Writes the dense routing weights
// moe_w[e][row_stride] (0 where the row does not use expert e) and expert_used[e].  Block = one row.
__global__ __launch_bounds__(256) void k_router(const float* xnorm, const float* h, const float* ssq, int ssq_groups, float inv_d,
                                                float eps, const float* gain, const float* __restrict__ router, int E, int topk,
                                                int d, int M, float* moe_w, int row_stride, int* expert_used) {
  __shared__ float sh[16];
  __shared__ float lg[64];
  const int r = blockIdx.x;
  float rstd = 1.f;
  if (!xnorm) {                                  // same class order as every other consumer of these partial sums
    if (threadIdx.x < 16) {
      float v[16];
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int g = (int)threadIdx.x + 16 * i;
        v[i] = g < ssq_groups ? ssq[g * 32 + r] : 0.f;
      }
      float a = 0.f;
#pragma unroll
      for (int i = 0; i < 16; ++i) a += v[i];
      sh[threadIdx.x] = a;
    }
    __syncthreads();
    float tot = 0.f;
    for (int c = 0; c < 16; ++c) tot += sh[c];
    rstd = 1.0f / sqrtf(tot * inv_d + eps);
    __syncthreads();                             // sh is reused by block_sum below
  }
  for (int e = 0; e < E; ++e) {
    float a = 0.f;
    for (int k = threadIdx.x; k < d; k += blockDim.x) {
      const float x = xnorm ? xnorm[(size_t)r * d + k] : h[(size_t)r * d + k] * rstd * gain[k];
      a += x * router[(size_t)e * d + k];
    }
    a = block_sum(a, sh);
    if (threadIdx.x == 0) lg[e] = a;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    int sel[4];
    float sv[4];
    for (int j = 0; j < topk; ++j) {
      float bv = -INFINITY; int bi = 0x7fffffff;
      for (int e = 0; e < E; ++e) {
        bool taken = false;
        for (int q = 0; q < j; ++q) taken |= (sel[q] == e);
        if (!taken) better(bv, bi, lg[e], e);
      }
      sel[j] = bi; sv[j] = bv;
    }
    float mx = sv[0], den = 0.f, p[4];
    for (int j = 0; j < topk; ++j) { p[j] = expf(sv[j] - mx); den += p[j]; }
    for (int e = 0; e < E; ++e) moe_w[(size_t)e * row_stride + r] = 0.f;
    for (int j = 0; j < topk; ++j) {
      moe_w[(size_t)sel[j] * row_stride + r] = p[j] / den;
      if (r < M) atomicOr(expert_used + sel[j], 1);
    }
  }
}

// ============================================================================ debug / test access
template <typename CT>
__global__ void k_read_kv_row(KVCache kv, int seq, int pos, float* kout, float* vout) {
  int n = kv.n_kv_heads * kv.head_dim;
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) {
    int kvh = i / kv.head_dim, d = i % kv.head_dim;
    size_t o = kv_offset(kv, seq, pos, kvh) + d;
    kout[i] = cache_load((const CT*)kv.k + o);
    vout[i] = cache_load((const CT*)kv.v + o);
  }
}

// Profiling: adds the number of experts at least one row selected (flags set by k_router) to a running total.
__global__ void k_count_used(const int* expert_used, int E, int* total) {
  if (threadIdx.x == 0 && blockIdx.x == 0) {
    int n = 0;
    for (int e = 0; e < E; ++e) n += expert_used[e] != 0;
    *total += n;
  }
}

__global__ void k_fill_u32(uint32_t* p, uint32_t v, size_t n) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = v;
}
