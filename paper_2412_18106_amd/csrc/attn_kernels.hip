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
//    holding two (K, V) block pairs; the next block is in flight to registers
//    while the current one is consumed.
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

// ---- global -> register -> LDS staging of one (K, V) block pair -------------
// Thread t moves 16-byte chunk (row = t/16 + 16e, col = t%16) for e = 0..7 of both tiles.
// K rows are stored with their 16-byte chunks XOR-ed by (swap23(row) & 15), V rows by
// ((row & 3) << 2): both reads below are then spread over all LDS banks.
struct Staged {
  uint4 k[8];
  uint4 v[8];
};

__device__ __forceinline__ void load_block(Staged& st, const RunParams& p, int64_t phys, int kvh, int tid) {
  const int64_t base = phys * p.kv_bs + (int64_t)kvh * p.kv_hs;
  const int col = tid & 15;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const int row = (tid >> 4) + 16 * e;
    const int64_t off = base + (int64_t)row * p.kv_ts + col * 8;
    st.k[e] = *reinterpret_cast<const uint4*>(p.k + off);
    st.v[e] = *reinterpret_cast<const uint4*>(p.v + off);
  }
}

__device__ __forceinline__ void store_block(const Staged& st, unsigned char* kt, unsigned char* vt, int tid) {
  const int col = tid & 15;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const int row = (tid >> 4) + 16 * e;
    *reinterpret_cast<uint4*>(kt + row * 256 + ((col ^ (swap23(row) & 15)) << 4)) = st.k[e];
    *reinterpret_cast<uint4*>(vt + row * 256 + ((col ^ ((row & 3) << 2)) << 4)) = st.v[e];
  }
}

// ---- one work unit ------------------------------------------------------------
__device__ void process_unit(const RunParams& p, const XyDevUnit& u, unsigned char* smem) {
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int col = lane & 31;        // which query row of a 32-row tile this lane owns
  const int half = lane >> 5;       // which 8-key half of every 16-key MFMA step

  const XyDevSeq sq = p.seqs[u.seq];
  const int hc = u.head_count;
  const int rows = u.q_count * hc;
  const bool small = rows <= 64;
  const bool tree = (u.flags >> 2) & 1;
  const int kvh = u.head_begin / p.group;
  const int ctx = sq.ctx_len;
  const int wpr = (sq.q_len + 31) >> 5;

  const int row_base = small ? 0 : 64 * wave;
  const int step_first = small ? wave : 0;
  const int step_inc = small ? 4 : 1;
  const int rows_here = rows - row_base;                       // may be <= 0
  const int ntiles = rows_here <= 0 ? 0 : (rows_here > 32 ? 2 : 1);

  // per-lane row bookkeeping for the two 32-row tiles
  int lim[2];                 // causal: number of visible keys; 0 for padding rows
  int tok[2];                 // token index inside the sequence
  bool valid[2];
  const uint16_t* qrow[2];
#pragma unroll
  for (int rt = 0; rt < 2; ++rt) {
    const int rho = row_base + 32 * rt + col;
    valid[rt] = rho < rows;
    const int tl = rho / hc, hl = rho - tl * hc;
    tok[rt] = u.q_begin + tl;
    lim[rt] = valid[rt] ? ctx + tok[rt] + 1 : 0;
    qrow[rt] = p.q + (int64_t)(sq.token_start + tok[rt]) * p.q_ts + (int64_t)(u.head_begin + hl) * p.q_hs;
  }
  // smallest causal limit among this wavefront's rows (rows are token-major, so it is the first row's)
  const int first_tok = u.q_begin + row_base / hc;
  const int mask_from = tree ? ctx : ctx + first_tok + 1;       // keys >= mask_from need a per-element test
  const int key_end = tree ? ctx + sq.q_len : ctx + u.q_begin + u.q_count;   // exclusive

  // Q fragments: B operand of S^T = K Q^T, lane (col, half) holds d = 16*ks + 8*half .. +7 of its row
  bf16x8 qf[2][8];
#pragma unroll
  for (int rt = 0; rt < 2; ++rt)
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      uint4 raw = make_uint4(0, 0, 0, 0);
      if (valid[rt]) raw = *reinterpret_cast<const uint4*>(qrow[rt] + 16 * ks + 8 * half);
      qf[rt][ks] = __builtin_bit_cast(bf16x8, raw);
    }

  f32x16 oacc[2][4];          // O^T accumulators: [row tile][32-wide d tile]
#pragma unroll
  for (int rt = 0; rt < 2; ++rt)
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int v = 0; v < 16; ++v) oacc[rt][dt][v] = 0.f;
  float m_ref[2] = {-INFINITY, -INFINITY};   // reference max (raw score units), may lag the true max
  float l_part[2] = {0.f, 0.f};              // this lane's share of the running sum

  const int32_t* table = p.block_table + (int64_t)u.seq * p.max_blocks;
  const int nblk = u.kv_end - u.kv_begin;

  Staged st;
  __syncthreads();            // previous unit's readers are done with LDS
  load_block(st, p, table[u.kv_begin], kvh, tid);
  store_block(st, smem, smem + kTileBytes, tid);
  __syncthreads();

  for (int ib = 0; ib < nblk; ++ib) {
    const int b = u.kv_begin + ib;
    unsigned char* kt = smem + (ib & 1) * 2 * kTileBytes;
    unsigned char* vt = kt + kTileBytes;
    const bool more = ib + 1 < nblk;
    if (more) load_block(st, p, table[b + 1], kvh, tid);

    const int j0 = b * kB;
    const int nvalid = min(kB, key_end - j0);      // keys of this block any row may see

    if (ntiles > 0) {
      for (int step = step_first; step < 4; step += step_inc) {
        const int kk = 32 * step;
        if (kk >= nvalid) break;
        // ---- S^T = K Q^T for 32 keys x (32 * ntiles) rows --------------------
        f32x16 s[2];
#pragma unroll
        for (int rt = 0; rt < 2; ++rt)
#pragma unroll
          for (int v = 0; v < 16; ++v) s[rt][v] = 0.f;
        const int krow = kk + swap23(col);
        const unsigned char* kbase = kt + krow * 256;
        const int kswz = col & 15;                 // == swap23(krow) & 15
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
          const bf16x8 kf = *reinterpret_cast<const bf16x8*>(kbase + (((2 * ks + half) ^ kswz) << 4));
          s[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[0][ks], s[0], 0, 0, 0);
          if (ntiles > 1) s[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[1][ks], s[1], 0, 0, 0);
        }
        // register v of s[rt] is key j0 + kk + 16*(v>>3) + 8*half + (v&7) for this lane's row
        const bool need_mask = j0 + kk + 32 > mask_from;
#pragma unroll
        for (int rt = 0; rt < 2; ++rt) {
          if (rt >= ntiles) break;
          if (need_mask) {
            if (!tree) {
#pragma unroll
              for (int v = 0; v < 16; ++v) {
                const int j = j0 + kk + 16 * (v >> 3) + 8 * half + (v & 7);
                if (j >= lim[rt]) s[rt][v] = -INFINITY;
              }
            } else {
              const uint32_t* mrow = p.masks + sq.mask_off + (int64_t)tok[rt] * wpr;
#pragma unroll
              for (int v = 0; v < 16; ++v) {
                const int j = j0 + kk + 16 * (v >> 3) + 8 * half + (v & 7);
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
          float mx = s[rt][0];
#pragma unroll
          for (int v = 1; v < 16; ++v) mx = fmaxf(mx, s[rt][v]);
          mx = fmaxf(mx, other_half(mx));
          const bool bump = mx * p.c > m_ref[rt] * p.c + kLazyRescale || (m_ref[rt] == -INFINITY && mx > -INFINITY);
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
        bf16x8 pf[2][2];
#pragma unroll
        for (int rt = 0; rt < 2; ++rt)
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
            oacc[0][dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vfb, pf[0][t], oacc[0][dt], 0, 0, 0);
            if (ntiles > 1) oacc[1][dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vfb, pf[1][t], oacc[1][dt], 0, 0, 0);
          }
        }
      }
    }
    if (more) store_block(st, smem + ((ib + 1) & 1) * 2 * kTileBytes, smem + ((ib + 1) & 1) * 2 * kTileBytes + kTileBytes, tid);
    __syncthreads();
  }

  // ---- finish: combine the two lane halves' sums --------------------------------
  float l_tot[2];
#pragma unroll
  for (int rt = 0; rt < 2; ++rt) l_tot[rt] = l_part[rt] + other_half(l_part[rt]);

  if (small) {
    // Four wavefronts hold partial states over disjoint keys of the same rows: merge through LDS.
    float* obuf = reinterpret_cast<float*>(smem);              // [4 waves][ntiles*32 rows][128] fp32
    float* mbuf = reinterpret_cast<float*>(smem + 4 * kTileBytes);   // [4][64] m (log2 units)
    float* lbuf = mbuf + 256;                                  // [4][64] l scaled to the common max
    const int nrow_pad = ntiles * 32;
#pragma unroll
    for (int rt = 0; rt < 2; ++rt)
      if (rt < ntiles && half == 0) mbuf[wave * 64 + 32 * rt + col] = (m_ref[rt] == -INFINITY) ? -INFINITY : m_ref[rt] * p.c;
    __syncthreads();
#pragma unroll
    for (int rt = 0; rt < 2; ++rt) {
      if (rt >= ntiles) break;
      const int r = 32 * rt + col;
      const float mstar = fmaxf(fmaxf(mbuf[r], mbuf[64 + r]), fmaxf(mbuf[128 + r], mbuf[192 + r]));
      const float mine = (m_ref[rt] == -INFINITY) ? -INFINITY : m_ref[rt] * p.c;
      const float f = (mine == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(mine - mstar);
      if (half == 0) lbuf[wave * 64 + r] = l_tot[rt] * f;
#pragma unroll
      for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int d = 32 * dt + 8 * (v >> 2) + 4 * half + (v & 3);
          obuf[(wave * nrow_pad + r) * kD + d] = oacc[rt][dt][v] * f;
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
    for (int rt = 0; rt < 2; ++rt) {
      if (rt >= ntiles || !valid[rt]) continue;
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
    process_unit(p, u, smem);
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
