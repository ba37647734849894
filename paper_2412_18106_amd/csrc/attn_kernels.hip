// Attention meta-kernel for gfx950: a persistent kernel in which every workgroup
// walks its own list of (Q tile x KV block range) work units, plus the merge
// pass for K/V-split units.
//
// What is computed (paper section 4): per unit, S = scale * Q K^T over the KV
// blocks the unit visits, a row softmax restricted to the visible keys
// (causal bound of section 4.2.2, tree corner of section 4.1.2, tail of the
// last block neutralised as in section 5.2) and O = P V, in the K/V-split
// form with running max / sum (the Update stage of section 4.2.1).  The unit's
// origin (prefill, decode, verify) does not change the code path: only its row
// count does.
//
// How it is laid out on CDNA4 (this design, not the paper's):
//  * 256 threads = 4 wavefronts per workgroup, one workgroup per CU, 128 KB LDS
//    holding two (K, V) block pairs; the next block streams from HBM straight
//    into LDS (no staging registers) while the current one is consumed.
//  * Scores are produced transposed, S^T = K Q^T, with the 32x32x16 bf16 MFMA:
//    a lane then owns ONE query row (max / sum need one cross-lane exchange), the
//    accumulator registers of S^T are already the B operand of O^T += V^T P^T,
//    and rescaling O^T is one scalar per lane.
//  * V^T fragments come from the row-major V tile in LDS through the
//    transposing LDS read (ds_read_b64_tr_b16).
//  * rows = tokens x heads of one KV head (GQA sharing): a unit with more than
//    64 rows gives each wavefront 64 rows and every key; a unit with up to 64
//    rows (decode, short verify) gives each wavefront all rows and a quarter of
//    each block's keys, merged through LDS at the end.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>

#include "plan_internal.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr int kD = 128;          // head dim
constexpr int kB = 128;          // tokens per KV block
constexpr int kTileBytes = kB * kD * 2;   // one K or V tile of one KV head
constexpr int kThreads = 256;
constexpr float kLazyRescale = 8.0f;      // log2 units the running max may lag behind

struct RunParams {
  const XyDevUnit* units;
  const int32_t* worker_offsets;
  const XyDevSeq* seqs;
  const uint16_t* q;
  const uint16_t* k;
  const uint16_t* v;
  const int32_t* block_table;
  const uint32_t* masks;
  uint16_t* out;
  float* ws;
  int64_t q_ts, q_hs, kv_bs, kv_hs, kv_ts, o_ts, o_hs;
  int32_t max_blocks, group, num_workers;
  float c;      // softmax_scale * log2(e)
};

__device__ __forceinline__ int swap23(int i) {   // exchange bits 2 and 3
  return (i & ~12) | ((i & 4) << 1) | ((i & 8) >> 1);
}

// value held by the lane 32 places away
__device__ __forceinline__ float other_half(float x) {
  unsigned u = __builtin_bit_cast(unsigned, x);
  auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  // r[0]: lanes < 32 keep own, lanes >= 32 get lane-32's; r[1]: lanes < 32 get lane+32's, lanes >= 32 keep own
  unsigned o = (threadIdx.x & 32) ? r[0] : r[1];
  return __builtin_bit_cast(float, o);
}

__device__ __forceinline__ unsigned pack_bf16(float a, float b) {
  typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
  bf16x2 p = {(__bf16)a, (__bf16)b};
  return __builtin_bit_cast(unsigned, p);
}

// ---- global -> LDS staging of one (K, V) block pair ---------------------------
// Each wavefront instruction moves 64 x 16 bytes straight into 1 KB of LDS (4 rows of a tile)
// without passing through registers.  LDS slot (row, p) of a tile receives the 16-byte chunk
// p ^ swz(row) of that row; K uses swz = swap23(row) & 15, V uses swz = (row & 3) << 2, which
// spreads the fragment reads below over all LDS banks.
__device__ __forceinline__ void load_block_async(const RunParams& p, int64_t phys, int kvh, unsigned char* kt,
                                                 unsigned char* vt, int wave, int lane) {
  const int64_t base = phys * p.kv_bs + (int64_t)kvh * p.kv_hs;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const int grp = wave * 8 + e;                 // 4 consecutive rows
    const int row = 4 * grp + (lane >> 4);
    const int pos = lane & 15;
    const int64_t roff = base + (int64_t)row * p.kv_ts;
    const uint16_t* ksrc = p.k + roff + ((pos ^ (swap23(row) & 15)) << 3);
    const uint16_t* vsrc = p.v + roff + ((pos ^ ((row & 3) << 2)) << 3);
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)ksrc,
                                     (__attribute__((address_space(3))) void*)(kt + grp * 1024), 16, 0, 0);
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)vsrc,
                                     (__attribute__((address_space(3))) void*)(vt + grp * 1024), 16, 0, 0);
  }
}

__device__ __forceinline__ void wait_loads_and_sync() {
  __builtin_amdgcn_s_waitcnt(0x0F70);     // vmcnt(0): this wavefront's LDS-direct loads have landed
  __syncthreads();
}

// ---- one work unit ------------------------------------------------------------
// NT = number of 32-row tiles this wavefront owns (1 or 2).
template <int NT>
__device__ __forceinline__ void process_unit(const RunParams& p, const XyDevUnit& u, const XyDevSeq& sq,
                                             unsigned char* smem, const bool small) {
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int col = lane & 31;        // which query row of a 32-row tile this lane owns
  const int half = lane >> 5;       // which 8-key half of every 16-key MFMA step

  const int hc = u.head_count;
  const int rows = u.q_count * hc;
  const bool tree = (u.flags >> 2) & 1;
  const int kvh = u.head_begin / p.group;
  const int ctx = sq.ctx_len;
  const int wpr = (sq.q_len + 31) >> 5;

  const int row_base = small ? 0 : 64 * wave;
  const int step_first = small ? wave : 0;
  const int step_inc = small ? 4 : 1;
  const bool active = row_base < rows;

  // per-lane row bookkeeping
  int lim[NT];                // causal: number of visible keys; 0 for padding rows
  int tok[NT];                // token index inside the sequence
  bool valid[NT];
  uint32_t mw0[NT], mw1[NT];  // tree corner bits 0..63 of this lane's row
  const uint16_t* qrow[NT];
#pragma unroll
  for (int rt = 0; rt < NT; ++rt) {
    const int rho = row_base + 32 * rt + col;
    valid[rt] = rho < rows;
    const int rc = min(rho, rows - 1) < 0 ? 0 : min(rho, rows - 1);   // padding lanes read a real row
    const int tl = rc / hc, hl = rc - tl * hc;
    tok[rt] = u.q_begin + tl;
    lim[rt] = valid[rt] ? ctx + tok[rt] + 1 : 0;
    qrow[rt] = p.q + (int64_t)(sq.token_start + tok[rt]) * p.q_ts + (int64_t)(u.head_begin + hl) * p.q_hs;
    mw0[rt] = mw1[rt] = 0;
    if (tree && valid[rt] && wpr <= 2) {
      const uint32_t* mrow = p.masks + sq.mask_off + (int64_t)tok[rt] * wpr;
      mw0[rt] = mrow[0];
      if (wpr > 1) mw1[rt] = mrow[1];
    }
  }
  // smallest causal limit among this wavefront's rows (rows are token-major, so it is the first row's)
  const int first_tok = u.q_begin + row_base / hc;
  const int mask_from = tree ? ctx : ctx + first_tok + 1;       // keys >= mask_from need a per-element test
  const int key_end = tree ? ctx + sq.q_len : ctx + u.q_begin + u.q_count;   // exclusive

  // Q fragments: B operand of S^T = K Q^T, lane (col, half) holds d = 16*ks + 8*half .. +7 of its row
  bf16x8 qf[NT][8];
#pragma unroll
  for (int rt = 0; rt < NT; ++rt)
#pragma unroll
    for (int ks = 0; ks < 8; ++ks)
      qf[rt][ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(qrow[rt] + 16 * ks + 8 * half));

  f32x16 oacc[NT][4];         // O^T accumulators: [row tile][32-wide d tile]
#pragma unroll
  for (int rt = 0; rt < NT; ++rt)
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int v = 0; v < 16; ++v) oacc[rt][dt][v] = 0.f;
  float m_ref[NT], l_part[NT];   // reference max (raw score units, may lag the true max); lane's share of the sum
#pragma unroll
  for (int rt = 0; rt < NT; ++rt) {
    m_ref[rt] = -INFINITY;
    l_part[rt] = 0.f;
  }

  const int32_t* table = p.block_table + (int64_t)u.seq * p.max_blocks;
  const int nblk = u.kv_end - u.kv_begin;

  __syncthreads();            // previous unit's readers are done with LDS
  load_block_async(p, table[u.kv_begin], kvh, smem, smem + kTileBytes, wave, lane);
  wait_loads_and_sync();

  for (int ib = 0; ib < nblk; ++ib) {
    const int b = u.kv_begin + ib;
    unsigned char* kt = smem + (ib & 1) * 2 * kTileBytes;
    unsigned char* vt = kt + kTileBytes;
    if (ib + 1 < nblk) {
      unsigned char* nk = smem + ((ib + 1) & 1) * 2 * kTileBytes;
      load_block_async(p, table[b + 1], kvh, nk, nk + kTileBytes, wave, lane);
    }
    const int j0 = b * kB;
    const int nvalid = min(kB, key_end - j0);      // keys of this block any row may see

    if (active) {
      for (int step = step_first; step < 4; step += step_inc) {
        const int kk = 32 * step;
        if (kk >= nvalid) break;
        // ---- S^T = K Q^T for 32 keys x (32 * NT) rows ------------------------
        f32x16 s[NT];
#pragma unroll
        for (int rt = 0; rt < NT; ++rt)
#pragma unroll
          for (int v = 0; v < 16; ++v) s[rt][v] = 0.f;
        const unsigned char* kbase = kt + (kk + swap23(col)) * 256;
        const int kswz = col & 15;                 // == swap23(row) & 15 of the row read here
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
          const bf16x8 kf = *reinterpret_cast<const bf16x8*>(kbase + (((2 * ks + half) ^ kswz) << 4));
#pragma unroll
          for (int rt = 0; rt < NT; ++rt) s[rt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[rt][ks], s[rt], 0, 0, 0);
        }
        // register v of s[rt] is key j0 + kk + 16*(v>>3) + 8*half + (v&7) for this lane's row
        const int jbase = j0 + kk + 8 * half;
        const bool need_mask = j0 + kk + 32 > mask_from;
#pragma unroll
        for (int rt = 0; rt < NT; ++rt) {
          if (need_mask) {
            if (!tree) {
#pragma unroll
              for (int v = 0; v < 16; ++v) {
                const int j = jbase + 16 * (v >> 3) + (v & 7);
                if (j >= lim[rt]) s[rt][v] = -INFINITY;
              }
            } else if (wpr <= 2) {
#pragma unroll
              for (int v = 0; v < 16; ++v) {
                const int j = jbase + 16 * (v >> 3) + (v & 7);
                const int sidx = j - ctx;          // corner column when >= 0
                const uint32_t w = (sidx & 32) ? mw1[rt] : mw0[rt];
                const bool bit = sidx < 64 && ((w >> (sidx & 31)) & 1u);
                const bool vis = valid[rt] && (sidx < 0 || bit);
                if (!vis) s[rt][v] = -INFINITY;
              }
            } else {
              const uint32_t* mrow = p.masks + sq.mask_off + (int64_t)tok[rt] * wpr;
#pragma unroll
              for (int v = 0; v < 16; ++v) {
                const int j = jbase + 16 * (v >> 3) + (v & 7);
                bool vis = valid[rt] && j < ctx;
                if (valid[rt] && j >= ctx && j < key_end) {
                  const int sidx = j - ctx;
                  vis = (mrow[sidx >> 5] >> (sidx & 31)) & 1u;
                }
                if (!vis) s[rt][v] = -INFINITY;
              }
            }
          }
          // ---- softmax with a lazily updated reference max -------------------
          float mx = fmaxf(s[rt][0], s[rt][1]);
#pragma unroll
          for (int v = 2; v < 16; ++v) mx = fmaxf(mx, s[rt][v]);
          mx = fmaxf(mx, other_half(mx));
          const bool bump = mx * p.c > m_ref[rt] * p.c + kLazyRescale;   // also true when m_ref is -inf and mx is not
          if (__any(bump)) {
            const float m_new = fmaxf(m_ref[rt], mx);
            const float alpha = (m_new == -INFINITY) ? 1.f : __builtin_amdgcn_exp2f((m_ref[rt] - m_new) * p.c);
            l_part[rt] *= alpha;
#pragma unroll
            for (int dt = 0; dt < 4; ++dt)
#pragma unroll
              for (int v = 0; v < 16; ++v) oacc[rt][dt][v] *= alpha;
            m_ref[rt] = m_new;
          }
          const float mc = (m_ref[rt] == -INFINITY) ? 0.f : m_ref[rt] * p.c;
          float sum = 0.f;
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const float e = __builtin_amdgcn_exp2f(s[rt][v] * p.c - mc);
            s[rt][v] = e;
            sum += e;
          }
          l_part[rt] += sum;
        }
        // ---- O^T += V^T P^T ---------------------------------------------------
        bf16x8 pf[NT][2];
#pragma unroll
        for (int rt = 0; rt < NT; ++rt)
#pragma unroll
          for (int t = 0; t < 2; ++t) {
            uint4 w;
            w.x = pack_bf16(s[rt][8 * t + 0], s[rt][8 * t + 1]);
            w.y = pack_bf16(s[rt][8 * t + 2], s[rt][8 * t + 3]);
            w.z = pack_bf16(s[rt][8 * t + 4], s[rt][8 * t + 5]);
            w.w = pack_bf16(s[rt][8 * t + 6], s[rt][8 * t + 7]);
            pf[rt][t] = __builtin_bit_cast(bf16x8, w);
          }
        // transposing read: a 16-lane group fetches 4 keys x 16 d; lane i16 supplies the address
        // of key (i16 / 4), d (4 * (i16 % 4)) and receives the 4 keys of d (i16).
        const int i16 = lane & 15;
        const int dsub = 16 * ((lane >> 4) & 1);
#pragma unroll
        for (int t = 0; t < 2; ++t) {
#pragma unroll
          for (int dt = 0; dt < 4; ++dt) {
            s16x8 vf;
#pragma unroll
            for (int hh = 0; hh < 2; ++hh) {
              const int key = kk + 16 * t + 8 * half + 4 * hh + (i16 >> 2);
              const int d0 = 32 * dt + dsub + 4 * (i16 & 3);
              const unsigned char* a = vt + key * 256 + ((((d0 >> 3)) ^ ((key & 3) << 2)) << 4) + ((d0 & 7) << 1);
              const s16x4 r = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                  (s16x4 __attribute__((address_space(3)))*)(a));
              vf[4 * hh + 0] = r[0];
              vf[4 * hh + 1] = r[1];
              vf[4 * hh + 2] = r[2];
              vf[4 * hh + 3] = r[3];
            }
            const bf16x8 vfb = __builtin_bit_cast(bf16x8, vf);
#pragma unroll
            for (int rt = 0; rt < NT; ++rt)
              oacc[rt][dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vfb, pf[rt][t], oacc[rt][dt], 0, 0, 0);
          }
        }
      }
    }
    wait_loads_and_sync();
  }

  // ---- finish: combine the two lane halves' sums --------------------------------
  float l_tot[NT];
#pragma unroll
  for (int rt = 0; rt < NT; ++rt) l_tot[rt] = l_part[rt] + other_half(l_part[rt]);

  if (small) {
    // Four wavefronts hold partial states over disjoint keys of the same rows: merge through LDS.
    float* obuf = reinterpret_cast<float*>(smem);              // [4 waves][NT*32 rows][128] fp32
    float* mbuf = reinterpret_cast<float*>(smem + 4 * kTileBytes);   // [4][64] m (log2 units)
    float* lbuf = mbuf + 256;                                  // [4][64] l scaled to the common max
    constexpr int nrow_pad = NT * 32;
#pragma unroll
    for (int rt = 0; rt < NT; ++rt)
      if (half == 0) mbuf[wave * 64 + 32 * rt + col] = (m_ref[rt] == -INFINITY) ? -INFINITY : m_ref[rt] * p.c;
    __syncthreads();
#pragma unroll
    for (int rt = 0; rt < NT; ++rt) {
      const int r = 32 * rt + col;
      const float mstar = fmaxf(fmaxf(mbuf[r], mbuf[64 + r]), fmaxf(mbuf[128 + r], mbuf[192 + r]));
      const float mine = (m_ref[rt] == -INFINITY) ? -INFINITY : m_ref[rt] * p.c;
      const float f = (mine == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(mine - mstar);
      if (half == 0) lbuf[wave * 64 + r] = l_tot[rt] * f;
#pragma unroll
      for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int a = 0; a < 4; ++a) {
          f32x4 x = {oacc[rt][dt][4 * a] * f, oacc[rt][dt][4 * a + 1] * f, oacc[rt][dt][4 * a + 2] * f,
                     oacc[rt][dt][4 * a + 3] * f};
          *reinterpret_cast<f32x4*>(obuf + (wave * nrow_pad + r) * kD + 32 * dt + 8 * a + 4 * half) = x;
        }
    }
    __syncthreads();
    // thread t sums 4 consecutive d of row (t / 32 + 8 * e)
    for (int r = tid >> 5; r < rows; r += 8) {
      const int d = (tid & 31) * 4;
      f32x4 acc = {0.f, 0.f, 0.f, 0.f};
      float l = 0.f, mstar = -INFINITY;
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const f32x4 x = *reinterpret_cast<const f32x4*>(obuf + (w * nrow_pad + r) * kD + d);
        acc += x;
        l += lbuf[w * 64 + r];
        mstar = fmaxf(mstar, mbuf[w * 64 + r]);
      }
      const int tl = r / hc, hl = r - tl * hc;
      if (u.ws_offset >= 0) {
        float* w = p.ws + u.ws_offset;
        *reinterpret_cast<f32x4*>(w + (int64_t)r * kD + d) = acc;
        if ((tid & 31) == 0) {
          w[(int64_t)rows * kD + r] = mstar;
          w[(int64_t)rows * kD + rows + r] = l;
        }
      } else {
        const float inv = l > 0.f ? 1.f / l : 0.f;
        uint16_t* o = p.out + (int64_t)(sq.token_start + u.q_begin + tl) * p.o_ts + (int64_t)(u.head_begin + hl) * p.o_hs + d;
        uint2 w2;
        w2.x = pack_bf16(acc[0] * inv, acc[1] * inv);
        w2.y = pack_bf16(acc[2] * inv, acc[3] * inv);
        *reinterpret_cast<uint2*>(o) = w2;
      }
    }
  } else {
#pragma unroll
    for (int rt = 0; rt < NT; ++rt) {
      if (!valid[rt]) continue;
      const int rho = row_base + 32 * rt + col;
      const int tl = rho / hc, hl = rho - tl * hc;
      if (u.ws_offset >= 0) {
        float* w = p.ws + u.ws_offset;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
          for (int a = 0; a < 4; ++a) {
            f32x4 x = {oacc[rt][dt][4 * a], oacc[rt][dt][4 * a + 1], oacc[rt][dt][4 * a + 2], oacc[rt][dt][4 * a + 3]};
            *reinterpret_cast<f32x4*>(w + (int64_t)rho * kD + 32 * dt + 8 * a + 4 * half) = x;
          }
        if (half == 0) {
          w[(int64_t)rows * kD + rho] = (m_ref[rt] == -INFINITY) ? -INFINITY : m_ref[rt] * p.c;
          w[(int64_t)rows * kD + rows + rho] = l_tot[rt];
        }
      } else {
        const float inv = l_tot[rt] > 0.f ? 1.f / l_tot[rt] : 0.f;
        uint16_t* o = p.out + (int64_t)(sq.token_start + u.q_begin + tl) * p.o_ts + (int64_t)(u.head_begin + hl) * p.o_hs;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
          for (int a = 0; a < 4; ++a) {
            uint2 w2;
            w2.x = pack_bf16(oacc[rt][dt][4 * a] * inv, oacc[rt][dt][4 * a + 1] * inv);
            w2.y = pack_bf16(oacc[rt][dt][4 * a + 2] * inv, oacc[rt][dt][4 * a + 3] * inv);
            *reinterpret_cast<uint2*>(o + 32 * dt + 8 * a + 4 * half) = w2;
          }
      }
    }
  }
}

__global__ __launch_bounds__(kThreads) void xy_attn_units_kernel(RunParams p) {
  __shared__ __attribute__((aligned(16))) unsigned char smem[4 * kTileBytes + 2048];
  // consecutive workgroup ids land on different XCDs; give each XCD a contiguous range of workers
  int worker = blockIdx.x;
  if ((p.num_workers & 7) == 0) worker = (blockIdx.x & 7) * (p.num_workers >> 3) + (blockIdx.x >> 3);
  const int begin = p.worker_offsets[worker], end = p.worker_offsets[worker + 1];
  for (int i = begin; i < end; ++i) {
    const XyDevUnit u = p.units[i];
    const XyDevSeq sq = p.seqs[u.seq];
    const int rows = u.q_count * u.head_count;
    if (rows <= 32)
      process_unit<1>(p, u, sq, smem, true);
    else
      process_unit<2>(p, u, sq, smem, rows <= 64);
  }
}

// Merge the partial states of one K/V-split family: O = sum_p 2^(m_p - m*) acc_p / sum_p 2^(m_p - m*) l_p.
__global__ __launch_bounds__(128) void xy_attn_merge_kernel(const xy_merge_item* items, const XyDevSeq* seqs,
                                                            const float* ws, uint16_t* out, int64_t o_ts,
                                                            int64_t o_hs) {
  const xy_merge_item it = items[blockIdx.x];
  const int rows = it.q_count * it.head_count;
  const int r = blockIdx.y;
  if (r >= rows) return;
  const int d = threadIdx.x;
  const int64_t slab = ((int64_t)rows * (kD + 2) + 3) & ~(int64_t)3;
  float mstar = -INFINITY;
  for (int s = 0; s < it.num_splits; ++s) mstar = fmaxf(mstar, ws[it.ws_offset + s * slab + (int64_t)rows * kD + r]);
  float num = 0.f, den = 0.f;
  for (int s = 0; s < it.num_splits; ++s) {
    const float* w = ws + it.ws_offset + s * slab;
    const float m = w[(int64_t)rows * kD + r];
    const float f = (m == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(m - mstar);
    num += f * w[(int64_t)r * kD + d];
    den += f * w[(int64_t)rows * kD + rows + r];
  }
  const float o = den > 0.f ? num / den : 0.f;
  const int tl = r / it.head_count, hl = r - tl * it.head_count;
  const XyDevSeq sq = seqs[it.seq];
  const __bf16 ob = (__bf16)o;
  out[(int64_t)(sq.token_start + it.q_begin + tl) * o_ts + (int64_t)(it.head_begin + hl) * o_hs + d] =
      __builtin_bit_cast(uint16_t, ob);
}

template <typename T>
int upload_vec(void** dst, const T* src, size_t n) {
  *dst = nullptr;
  const size_t bytes = (n ? n : 1) * sizeof(T);
  if (hipMalloc(dst, bytes) != hipSuccess) return XY_ERR_HIP;
  if (n && hipMemcpy(*dst, src, n * sizeof(T), hipMemcpyHostToDevice) != hipSuccess) return XY_ERR_HIP;
  return XY_OK;
}

}  // namespace

void xy_plan_free_device(xy_attn_plan* plan) {
  if (!plan || plan->device < 0) return;
  int cur = 0;
  (void)hipGetDevice(&cur);
  (void)hipSetDevice(plan->device);
  if (plan->d_units) (void)hipFree(plan->d_units);
  if (plan->d_offsets) (void)hipFree(plan->d_offsets);
  if (plan->d_seqs) (void)hipFree(plan->d_seqs);
  if (plan->d_merges) (void)hipFree(plan->d_merges);
  plan->d_units = plan->d_offsets = plan->d_seqs = plan->d_merges = nullptr;
  plan->device = -1;
  (void)hipSetDevice(cur);
}

extern "C" int xy_attn_plan_upload(xy_attn_plan* plan) {
  if (!plan) return XY_ERR_ARG;
  if (plan->device >= 0) return XY_OK;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return XY_ERR_HIP;
  std::vector<XyDevUnit> du(plan->units.size());
  for (size_t i = 0; i < du.size(); ++i) {
    const xy_work_unit& u = plan->units[i];
    du[i] = XyDevUnit{u.seq, u.head_begin, u.head_count, u.q_begin, u.q_count,
                      u.kv_block_begin, u.kv_block_end, u.kind_flags, u.ws_offset};
  }
  std::vector<XyDevSeq> ds(plan->num_seqs);
  for (int32_t i = 0; i < plan->num_seqs; ++i) {
    const xy_seq_desc& s = plan->descs[i];
    ds[i] = XyDevSeq{s.query_len, s.context_len, plan->token_start[i], s.mask_kind, s.mask_word_offset};
  }
  plan->device = dev;
  int rc = upload_vec(&plan->d_units, du.data(), du.size());
  if (!rc) rc = upload_vec(&plan->d_offsets, plan->worker_offsets.data(), plan->worker_offsets.size());
  if (!rc) rc = upload_vec(&plan->d_seqs, ds.data(), ds.size());
  if (!rc) rc = upload_vec(&plan->d_merges, plan->merges.data(), plan->merges.size());
  if (rc) {
    xy_plan_free_device(plan);
    return rc;
  }
  return XY_OK;
}

static int run_impl(int phases, xy_attn_plan* plan, const void* q, int64_t q_ts, int64_t q_hs, const void* k_cache,
                    const void* v_cache, int64_t kv_bs, int64_t kv_hs, int64_t kv_ts,
                    const int32_t* block_table, const uint32_t* tree_masks, void* out, int64_t o_ts,
                    int64_t o_hs, void* workspace, size_t workspace_bytes, float softmax_scale,
                    void* hip_stream) {
  if (!plan || !(phases & (XY_PHASE_UNITS | XY_PHASE_MERGE)) || (phases & ~(XY_PHASE_UNITS | XY_PHASE_MERGE)))
    return XY_ERR_ARG;
  if (plan->units.empty()) return XY_OK;
  if (!q || !k_cache || !v_cache || !block_table || !out) return XY_ERR_ARG;
  if (plan->has_tree && !tree_masks) return XY_ERR_ARG;
  if (!(softmax_scale > 0.f) || !std::isfinite(softmax_scale)) return XY_ERR_ARG;
  // 16-byte vector accesses: every stride a multiple of 8 elements, every base 16-byte aligned
  const int64_t strides[] = {q_ts, q_hs, kv_bs, kv_hs, kv_ts, o_ts, o_hs};
  for (int64_t s : strides)
    if (s < 0 || (s & 7)) return XY_ERR_ARG;
  if (q_hs < kD || kv_ts < kD || o_hs < kD) return XY_ERR_ARG;
  const uintptr_t ptrs[] = {(uintptr_t)q, (uintptr_t)k_cache, (uintptr_t)v_cache, (uintptr_t)out};
  for (uintptr_t a : ptrs)
    if (a & 15) return XY_ERR_ARG;
  const size_t need = (size_t)plan->workspace_floats * sizeof(float);
  if (need && (!workspace || workspace_bytes < need || ((uintptr_t)workspace & 15))) return XY_ERR_WORKSPACE;
  if (int rc = xy_attn_plan_upload(plan)) return rc;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev != plan->device) return XY_ERR_ARG;

  RunParams p;
  p.units = static_cast<const XyDevUnit*>(plan->d_units);
  p.worker_offsets = static_cast<const int32_t*>(plan->d_offsets);
  p.seqs = static_cast<const XyDevSeq*>(plan->d_seqs);
  p.q = static_cast<const uint16_t*>(q);
  p.k = static_cast<const uint16_t*>(k_cache);
  p.v = static_cast<const uint16_t*>(v_cache);
  p.block_table = block_table;
  p.masks = tree_masks;
  p.out = static_cast<uint16_t*>(out);
  p.ws = static_cast<float*>(workspace);
  p.q_ts = q_ts; p.q_hs = q_hs; p.kv_bs = kv_bs; p.kv_hs = kv_hs; p.kv_ts = kv_ts; p.o_ts = o_ts; p.o_hs = o_hs;
  p.max_blocks = plan->cfg.max_blocks_per_seq;
  p.group = plan->cfg.num_q_heads / plan->cfg.num_kv_heads;
  p.num_workers = plan->cfg.num_workers;
  p.c = softmax_scale * 1.4426950408889634f;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  if (phases & XY_PHASE_UNITS) {
    hipLaunchKernelGGL(xy_attn_units_kernel, dim3(plan->cfg.num_workers), dim3(kThreads), 0, stream, p);
    if (hipGetLastError() != hipSuccess) return XY_ERR_HIP;
  }
  if ((phases & XY_PHASE_MERGE) && !plan->merges.empty()) {
    hipLaunchKernelGGL(xy_attn_merge_kernel, dim3((unsigned)plan->merges.size(), (unsigned)plan->max_merge_rows),
                       dim3(128), 0, stream, static_cast<const xy_merge_item*>(plan->d_merges), p.seqs,
                       static_cast<const float*>(workspace), p.out, o_ts, o_hs);
    if (hipGetLastError() != hipSuccess) return XY_ERR_HIP;
  }
  return XY_OK;
}

extern "C" int xy_attn_run(xy_attn_plan* plan, const void* q, int64_t q_ts, int64_t q_hs, const void* k_cache,
                           const void* v_cache, int64_t kv_bs, int64_t kv_hs, int64_t kv_ts,
                           const int32_t* block_table, const uint32_t* tree_masks, void* out, int64_t o_ts,
                           int64_t o_hs, void* workspace, size_t workspace_bytes, float softmax_scale,
                           void* hip_stream) {
  return run_impl(XY_PHASE_UNITS | XY_PHASE_MERGE, plan, q, q_ts, q_hs, k_cache, v_cache, kv_bs, kv_hs, kv_ts,
                  block_table, tree_masks, out, o_ts, o_hs, workspace, workspace_bytes, softmax_scale, hip_stream);
}

extern "C" int xy_attn_run_phase(int phases, xy_attn_plan* plan, const void* q, int64_t q_ts, int64_t q_hs,
                                 const void* k_cache, const void* v_cache, int64_t kv_bs, int64_t kv_hs,
                                 int64_t kv_ts, const int32_t* block_table, const uint32_t* tree_masks,
                                 void* out, int64_t o_ts, int64_t o_hs, void* workspace, size_t workspace_bytes,
                                 float softmax_scale, void* hip_stream) {
  return run_impl(phases, plan, q, q_ts, q_hs, k_cache, v_cache, kv_bs, kv_hs, kv_ts, block_table, tree_masks,
                  out, o_ts, o_hs, workspace, workspace_bytes, softmax_scale, hip_stream);
}
