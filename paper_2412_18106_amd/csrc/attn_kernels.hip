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
//  * 512 threads = 8 wavefronts per workgroup (two per SIMD, at most 256 registers
//    each), one workgroup per CU, 128 KB LDS holding two (K, V) block pairs; the
//    next block streams from HBM straight into LDS (no staging registers) while
//    the current one is consumed.
//  * Scores are produced transposed, S^T = K Q^T, with the 32x32x16 bf16 MFMA:
//    a lane then owns ONE query row (max / sum need one cross-lane exchange), the
//    accumulator registers of S^T are already the B operand of O^T += V^T P^T,
//    and rescaling O^T is one scalar per lane.
//  * V^T fragments come from the row-major V tile in LDS through the
//    transposing LDS read (ds_read_b64_tr_b16).
//  * rows = tokens x heads of one KV head (GQA sharing): a unit with more than
//    32 rows gives each wavefront 32 rows and every key, the wavefronts sharing
//    the block's tiles; a unit with up to 32 rows (decode, short verify) is
//    processed by a single wavefront streaming 32-key slices through a private
//    LDS ring, so a CU has eight such units in flight and no barrier between them.
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
constexpr int kB = 128;          // keys per K/V tile (one or more pages of the block table)
constexpr int kTileBytes = kB * kD * 2;   // one K or V tile of one KV head
constexpr int kThreads = 512;        // 8 wavefronts: two per SIMD
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
  int32_t page_shift, page_mask;     // log2 of the tokens per block-table entry (page), and that size - 1
  float c;      // softmax_scale * log2(e)
};

// Read-only tables (units, sequences, block table, the kernel arguments themselves) are read through
// the constant address space: with a uniform address such a load is a scalar load, which neither
// occupies a vector register nor shares the in-order counter of the LDS-direct K/V stream.
#define XY_CONST __attribute__((address_space(4)))
template <typename T>
__device__ __forceinline__ const XY_CONST T* as_const(const T* ptr) {
  return (const XY_CONST T*)ptr;
}

template <typename T>     // whole-struct copy out of a read-only table, word by word
__device__ __forceinline__ T load_const(const T* ptr) {
  static_assert(sizeof(T) % 4 == 0, "word-sized records only");
  T out;
  const XY_CONST uint32_t* src = (const XY_CONST uint32_t*)ptr;
  uint32_t* dst = reinterpret_cast<uint32_t*>(&out);
#pragma unroll
  for (unsigned i = 0; i < sizeof(T) / 4; ++i) dst[i] = src[i];
  return out;
}

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

// maximum of x over this lane and the lane 32 places away
__device__ __forceinline__ float max_both_halves(float x) {
  unsigned u = __builtin_bit_cast(unsigned, x);
  auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);   // r[0] = lower half's x, r[1] = upper half's x
  return fmaxf(__builtin_bit_cast(float, (unsigned)r[0]), __builtin_bit_cast(float, (unsigned)r[1]));
}

__device__ __forceinline__ unsigned pack_bf16(float a, float b) {
  typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
  bf16x2 p = {(__bf16)a, (__bf16)b};
  return __builtin_bit_cast(unsigned, p);
}

// ---- global -> LDS staging -------------------------------------------------------
// One wavefront instruction moves 64 x 16 bytes straight into 1 KB of LDS (4 rows of a tile)
// without passing through registers.  LDS slot (row, p) of a tile receives the 16-byte chunk
// p ^ swz(row) of that row; K uses swz = swap23(row) & 15, V uses swz = (row & 3) << 2, which
// spreads the fragment reads below over all LDS banks.  Both depend on the low 4 bits of the
// row only, so any 32-row slice of a tile is laid out the same way.
// The global address of lane l in instruction e is (uniform) tile + (row0 + 4e) rows, plus a
// per-lane 32-bit byte offset that depends on e only through e % 4: five registers per lane in all.
struct DmaOffsets {
  unsigned k[4];    // (l / 16) rows + swizzled chunk of K for e % 4
  unsigned v;       // the same for V (its swizzle does not depend on e)
};

__device__ __forceinline__ DmaOffsets make_dma_offsets(int lane, int64_t kv_ts) {
  DmaOffsets d;
  const int sub = lane >> 4, pos = lane & 15;
  const unsigned rowpart = (unsigned)(sub * kv_ts * 2);
#pragma unroll
  for (int j = 0; j < 4; ++j) d.k[j] = rowpart + ((pos ^ (swap23(4 * j + sub) & 15)) << 4);
  d.v = rowpart + ((pos ^ ((sub & 3) << 2)) << 4);
  return d;
}

template <int NGROUPS>   // NGROUPS x 4 rows, starting at row0 (a multiple of 16), into lds_k / lds_v
__device__ __forceinline__ void load_rows_async(const uint16_t* kg, const uint16_t* vg, int64_t kv_ts, int row0,
                                                unsigned char* lds_k, unsigned char* lds_v, const DmaOffsets& dof,
                                                const bool want_k, const bool want_v) {
#pragma unroll
  for (int e = 0; e < NGROUPS; ++e) {
    const int64_t rows = (int64_t)(row0 + 4 * e) * kv_ts;          // uniform
    if (want_k)
      __builtin_amdgcn_global_load_lds(
          (const __attribute__((address_space(1))) void*)(reinterpret_cast<const char*>(kg + rows) + (size_t)dof.k[e & 3]),
          (__attribute__((address_space(3))) void*)(lds_k + e * 1024), 16, 0, 0);
    if (want_v)
      __builtin_amdgcn_global_load_lds(
          (const __attribute__((address_space(1))) void*)(reinterpret_cast<const char*>(vg + rows) + (size_t)dof.v),
          (__attribute__((address_space(3))) void*)(lds_v + e * 1024), 16, 0, 0);
  }
}

// ---- LDS fragment reads -----------------------------------------------------------
// The fragment reads are issued as inline assembly and waited for by hand.  The compiler cannot
// tell that a read of one LDS buffer does not depend on an LDS-direct load still in flight to
// ANOTHER buffer, and would drain every outstanding K/V load before each read; issued this way
// the K/V stream stays in flight while the current block is consumed.  Every read is waited for
// (lds_wait) before its registers are used and before its buffer is refilled.
__device__ __forceinline__ unsigned lds_addr(const void* ptr) {
  return (unsigned)(size_t)((__attribute__((address_space(3))) const unsigned char*)ptr);
}

template <int OFF>
__device__ __forceinline__ bf16x8 lds_read_b128(unsigned addr) {
  bf16x8 r;
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(r) : "v"(addr), "n"(OFF) : "memory");
  return r;
}

template <int OFF>
__device__ __forceinline__ s16x4 lds_read_tr16_b64(unsigned addr) {
  s16x4 r;
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(r) : "v"(addr), "n"(OFF) : "memory");
  return r;
}

// wait until at most N of this wavefront's LDS reads are outstanding; the operands tie the wait
// to the registers it protects, so no use can be scheduled above it
template <int N>
__device__ __forceinline__ void lds_wait(bf16x8& a, bf16x8& b, bf16x8& c, bf16x8& d) {
  asm volatile("s_waitcnt lgkmcnt(%4)" : "+v"(a), "+v"(b), "+v"(c), "+v"(d) : "n"(N) : "memory");
}

// Per-lane byte offsets of the fragments inside any 32-row slice of a K / V tile.
struct LaneOffsets {
  unsigned k[8];   // K fragment ks: row swap23(col), 16-byte chunk (2*ks + half) ^ (col & 15)
  unsigned v[4];   // V^T fragment of d tile dt for keys 8*half + (i16 >> 2); add (16*t + 4*hh) * 256
};

__device__ __forceinline__ LaneOffsets make_lane_offsets(int lane) {
  LaneOffsets lo;
  const int col = lane & 31, half = lane >> 5, i16 = lane & 15, dsub = 16 * ((lane >> 4) & 1);
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) lo.k[ks] = swap23(col) * 256 + (((2 * ks + half) ^ (col & 15)) << 4);
#pragma unroll
  for (int dt = 0; dt < 4; ++dt) {
    const int key = 8 * half + (i16 >> 2);
    const int d0 = 32 * dt + dsub + 4 * (i16 & 3);
    lo.v[dt] = key * 256 + (((d0 >> 3) ^ ((key & 3) << 2)) << 4) + ((d0 & 7) << 1);
  }
  return lo;
}

// s_waitcnt vmcnt(N) only (gfx9 encoding: vmcnt in bits 3:0 and 15:14, expcnt 6:4, lgkmcnt 11:8)
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (15 << 8));
}

// Element offset (inside the K or V cache, before the KV head is added) of key row j of a sequence:
// page seq_table[j / page size], slot j % page size (paper section 4.1.1).  Sixteen consecutive rows
// starting at a multiple of 16 always share a page (pages hold 16, 32, 64 or 128 tokens).  Rows past
// the sequence's last page are never visible; they are redirected to the last page so that whatever
// lands in LDS for them is ordinary finite cache content.
__device__ __forceinline__ int64_t kv_row_offset(const XY_CONST int32_t* seq_table, int j, int last_page,
                                                 const RunParams& p) {
  const int page = min(j >> p.page_shift, last_page);
  return (int64_t)seq_table[page] * p.kv_bs + (int64_t)(j & p.page_mask) * p.kv_ts;
}

// ---- per-lane description of the query rows a wavefront owns -------------------------
template <int NT>
struct Rows {
  int lim[NT];                // causal: number of visible keys; 0 for padding rows
  int tok[NT];                // token index inside the sequence
  bool valid[NT];
  uint32_t mw0[NT], mw1[NT];  // tree corner bits 0..63 of this lane's row (a tree has at most 64 tokens)
};

struct UnitCtx {
  int hc, rows, kvh, ctx, wpr, key_end;
  bool tree;
};

__device__ __forceinline__ UnitCtx make_ctx(const RunParams& p, const XyDevUnit& u, const XyDevSeq& sq) {
  UnitCtx c;
  c.hc = u.head_count;
  c.rows = u.q_count * u.head_count;
  c.kvh = u.head_begin / p.group;
  c.ctx = sq.ctx_len;
  c.wpr = (sq.q_len + 31) >> 5;
  c.tree = (u.flags >> 2) & 1;
  c.key_end = c.tree ? sq.ctx_len + sq.q_len : sq.ctx_len + u.q_begin + u.q_count;   // exclusive
  return c;
}

// Row bookkeeping and Q fragments (B operand of S^T = K Q^T: lane (col, half) holds
// d = 16*ks + 8*half .. +7 of its row).  Padding lanes read a real row; their results are dropped.
template <int NT>
__device__ __forceinline__ void setup_rows(const RunParams& p, const XyDevUnit& u, const XyDevSeq& sq,
                                           const UnitCtx& c, int row_base, int col, int half, Rows<NT>& r,
                                           bf16x8 (&qf)[NT][8]) {
#pragma unroll
  for (int rt = 0; rt < NT; ++rt) {
    const int rho = row_base + 32 * rt + col;
    r.valid[rt] = rho < c.rows;
    const int rc = max(0, min(rho, c.rows - 1));
    const int tl = rc / c.hc, hl = rc - tl * c.hc;
    r.tok[rt] = u.q_begin + tl;
    r.lim[rt] = r.valid[rt] ? c.ctx + r.tok[rt] + 1 : 0;
    const uint16_t* qrow =
        p.q + (int64_t)(sq.token_start + r.tok[rt]) * p.q_ts + (int64_t)(u.head_begin + hl) * p.q_hs;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks)
      qf[rt][ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(qrow + 16 * ks + 8 * half));
    r.mw0[rt] = r.mw1[rt] = 0;
    if (c.tree && r.valid[rt]) {
      const uint32_t* mrow = p.masks + sq.mask_off + (int64_t)r.tok[rt] * c.wpr;
      r.mw0[rt] = mrow[0];
      if (c.wpr > 1) r.mw1[rt] = mrow[1];
    }
  }
}

// ---- S^T = K Q^T for 32 keys x (32 * NT) rows -------------------------------------
// kaddr: LDS byte address of the first of the 32 key rows.  Register v of s[rt] is key
// 16*(v>>3) + 8*half + (v&7) of those 32 for this lane's row.
template <int NT>
__device__ __forceinline__ void qk_step(unsigned kaddr, const LaneOffsets& lo, const bf16x8 (&qf)[NT][8],
                                        f32x16 (&s)[NT]) {
  bf16x8 ka[4], kb[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) ka[ks] = lds_read_b128<0>(kaddr + lo.k[ks]);
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) kb[ks] = lds_read_b128<0>(kaddr + lo.k[4 + ks]);
#pragma unroll
  for (int rt = 0; rt < NT; ++rt)
#pragma unroll
    for (int v = 0; v < 16; ++v) s[rt][v] = 0.f;
  lds_wait<4>(ka[0], ka[1], ka[2], ka[3]);
#pragma unroll
  for (int ks = 0; ks < 4; ++ks)
#pragma unroll
    for (int rt = 0; rt < NT; ++rt) s[rt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[ks], qf[rt][ks], s[rt], 0, 0, 0);
  lds_wait<0>(kb[0], kb[1], kb[2], kb[3]);
#pragma unroll
  for (int ks = 0; ks < 4; ++ks)
#pragma unroll
    for (int rt = 0; rt < NT; ++rt)
      s[rt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kb[ks], qf[rt][4 + ks], s[rt], 0, 0, 0);
}

// ---- visibility: causal bound (section 4.2.2) or tree corner (section 4.1.2) ----------
template <int NT>
__device__ __forceinline__ void mask_step(const RunParams& p, const XyDevSeq& sq, const UnitCtx& c,
                                          const Rows<NT>& r, int jbase /* key of register 0 */, f32x16 (&s)[NT]) {
#pragma unroll
  for (int rt = 0; rt < NT; ++rt) {
    if (!c.tree) {
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int j = jbase + 16 * (v >> 3) + (v & 7);
        if (j >= r.lim[rt]) s[rt][v] = -INFINITY;
      }
    } else {                  // at most 64 speculative tokens: both mask words of the row are in registers
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int sidx = jbase + 16 * (v >> 3) + (v & 7) - c.ctx;   // corner column when >= 0
        const uint32_t w = (sidx & 32) ? r.mw1[rt] : r.mw0[rt];
        const bool bit = sidx < 64 && ((w >> (sidx & 31)) & 1u);
        if (!(r.valid[rt] && (sidx < 0 || bit))) s[rt][v] = -INFINITY;
      }
    }
  }
}

// ---- softmax + Update (section 4.2.1) with a lazily raised reference max -------------
// On return s holds the un-normalised probabilities 2^((score - m_ref) * c) <= 2^kLazyRescale.
template <int NT>
__device__ __forceinline__ void softmax_step(float cs, f32x16 (&s)[NT], float (&m_ref)[NT], float (&l_part)[NT],
                                             f32x16 (&oacc)[NT][4]) {
#pragma unroll
  for (int rt = 0; rt < NT; ++rt) {
    float mx = fmaxf(s[rt][0], s[rt][1]);
#pragma unroll
    for (int v = 2; v < 16; ++v) mx = fmaxf(mx, s[rt][v]);
    mx = fmaxf(mx, other_half(mx));
    const bool bump = mx * cs > m_ref[rt] * cs + kLazyRescale;   // also true when m_ref is -inf and mx is not
    if (__any(bump)) {
      const float m_new = fmaxf(m_ref[rt], mx);
      const float alpha = (m_new == -INFINITY) ? 1.f : __builtin_amdgcn_exp2f((m_ref[rt] - m_new) * cs);
      l_part[rt] *= alpha;
#pragma unroll
      for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int v = 0; v < 16; ++v) oacc[rt][dt][v] *= alpha;
      m_ref[rt] = m_new;
    }
    const float mc = (m_ref[rt] == -INFINITY) ? 0.f : m_ref[rt] * cs;
    float sum = 0.f;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const float e = __builtin_amdgcn_exp2f(s[rt][v] * cs - mc);
      s[rt][v] = e;
      sum += e;
    }
    l_part[rt] += sum;
  }
}

// ---- O^T += V^T P^T for the same 32 keys ---------------------------------------------
// The transposing read serves a 16-lane group with 4 keys x 16 d: lane i16 supplies the address
// of key (i16 / 4), d (4 * (i16 % 4)) and receives the 4 keys of d (i16).  v_fetch issues the
// sixteen reads of a step (it may run ahead of the softmax), pv_step waits for them.
struct VFrags {
  bf16x8 f[4];        // [32-wide d tile] for one 16-key half
};

template <int T>      // T = which 16-key half of the step
__device__ __forceinline__ void v_fetch(unsigned vaddr, const LaneOffsets& lo, VFrags& vf) {
#pragma unroll
  for (int dt = 0; dt < 4; ++dt) {
    const unsigned a = vaddr + lo.v[dt];
    const s16x4 r0 = lds_read_tr16_b64<T * 16 * 256>(a);
    const s16x4 r1 = lds_read_tr16_b64<T * 16 * 256 + 4 * 256>(a);
    s16x8 w;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      w[e] = r0[e];
      w[4 + e] = r1[e];
    }
    vf.f[dt] = __builtin_bit_cast(bf16x8, w);
  }
}

template <int NT>
__device__ __forceinline__ bf16x8 pack_p(const f32x16& s, int t) {
  uint4 w;
  w.x = pack_bf16(s[8 * t + 0], s[8 * t + 1]);
  w.y = pack_bf16(s[8 * t + 2], s[8 * t + 3]);
  w.z = pack_bf16(s[8 * t + 4], s[8 * t + 5]);
  w.w = pack_bf16(s[8 * t + 6], s[8 * t + 7]);
  return __builtin_bit_cast(bf16x8, w);
}

// O^T accumulators are updated strictly in place.  Written as assembly with the accumulator tied to
// the destination: through the builtin the register allocator keeps migrating the 64 accumulator
// registers between two homes and pays 64 register moves per step.  The compiler does not know this
// is an MFMA, so the wait states it would insert before the result is read are provided by hand:
// inside the loop the next reader is hundreds of cycles away (after the next step's QK MFMAs), and
// after the loop mfma_results_ready() pads before the epilogue reads the accumulators.
template <bool FIRST_OF_GROUP>
__device__ __forceinline__ void mfma_acc(f32x16& acc, const bf16x8& a, const bf16x8& b) {
  // Wait states between a vector-ALU write of an operand (the packed P fragment, a rescaled
  // accumulator) and the MFMA reading it: five before the first MFMA of a group of four, two before
  // the others.  volatile keeps the issue order of the group, so two MFMAs on one accumulator stay
  // four instructions apart.
  if (FIRST_OF_GROUP)
    asm volatile("s_nop 4\n\tv_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(acc) : "v"(a), "v"(b));
  else
    asm volatile("s_nop 1\n\tv_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(acc) : "v"(a), "v"(b));
}
__device__ __forceinline__ void mfma_results_ready(f32x16& a, f32x16& b, f32x16& c, f32x16& d) {
  asm volatile("s_nop 7\n\ts_nop 7\n\ts_nop 7" : "+v"(a), "+v"(b), "+v"(c), "+v"(d));
}

// vf0 (keys 0..15 of the step) was fetched before the softmax; the fragments of keys 16..31 are
// fetched here, while the first four MFMAs run.
template <int NT>
__device__ __forceinline__ void pv_step(unsigned vaddr, const LaneOffsets& lo, VFrags& vf0, const f32x16 (&s)[NT],
                                        f32x16 (&oacc)[NT][4]) {
  VFrags vf1;
  v_fetch<1>(vaddr, lo, vf1);
  bf16x8 pf0[NT], pf1[NT];
#pragma unroll
  for (int rt = 0; rt < NT; ++rt) {
    pf0[rt] = pack_p<NT>(s[rt], 0);
    pf1[rt] = pack_p<NT>(s[rt], 1);
  }
  lds_wait<8>(vf0.f[0], vf0.f[1], vf0.f[2], vf0.f[3]);
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int rt = 0; rt < NT; ++rt) {
      if (dt == 0) mfma_acc<true>(oacc[rt][dt], vf0.f[dt], pf0[rt]);
      else mfma_acc<false>(oacc[rt][dt], vf0.f[dt], pf0[rt]);
    }
  lds_wait<0>(vf1.f[0], vf1.f[1], vf1.f[2], vf1.f[3]);
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int rt = 0; rt < NT; ++rt) {
      if (dt == 0) mfma_acc<true>(oacc[rt][dt], vf1.f[dt], pf1[rt]);
      else mfma_acc<false>(oacc[rt][dt], vf1.f[dt], pf1[rt]);
    }
}


// ---- wide units: the softmax split in two, so that its long part can share the issue stream with MFMAs ----
// Part 1: row max, lazy rescale; returns the exponent offset m_ref * c.
__device__ __forceinline__ float softmax_max(float cs, const f32x16& s, float& m_ref, float& l_part,
                                             f32x16 (&oacc)[1][4]) {
  float mx = fmaxf(s[0], s[1]);
#pragma unroll
  for (int v = 2; v < 16; ++v) mx = fmaxf(mx, s[v]);
  mx = max_both_halves(mx);
  const bool bump = mx * cs > m_ref * cs + kLazyRescale;   // also true when m_ref is -inf and mx is not
  if (__any(bump)) {
    const float m_new = fmaxf(m_ref, mx);
    const float alpha = (m_new == -INFINITY) ? 1.f : __builtin_amdgcn_exp2f((m_ref - m_new) * cs);
    l_part *= alpha;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int v = 0; v < 16; ++v) oacc[0][dt][v] *= alpha;
    m_ref = m_new;
  }
  return (m_ref == -INFINITY) ? 0.f : m_ref * cs;
}

// Part 2: the sixteen exponentials, the row-sum share and the bf16 packing of step t, written
// two scores at a time between the eight (dependent) MFMAs of S^T for step t + 1: the matrix pipe
// runs a 32-cycle MFMA while the vector ALU does an fma / exp2 / add / convert group of about
// the same length (the paper's cube / vector overlap of section 4.2.1, at instruction level).
template <bool WITH_QK>
__device__ __forceinline__ void exp_with_next_qk(float cs, float mc, const f32x16& s, float& l_part, bf16x8& pf0,
                                                 bf16x8& pf1, unsigned kaddr_next, const LaneOffsets& lo,
                                                 const bf16x8 (&qf)[1][8], f32x16& s_next) {
  bf16x8 ka[4], kb[4];
  if (WITH_QK) {
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) ka[ks] = lds_read_b128<0>(kaddr_next + lo.k[ks]);
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) kb[ks] = lds_read_b128<0>(kaddr_next + lo.k[4 + ks]);
    lds_wait<4>(ka[0], ka[1], ka[2], ka[3]);
  }
  typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
  const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
  unsigned packed[8];
  float sum0 = 0.f, sum1 = 0.f;    // the row sum adds the ROUNDED probabilities, two per instruction
  f32x16 acc;
#pragma unroll
  for (int v = 0; v < 16; ++v) acc[v] = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    if (WITH_QK) {
      if (i == 4) lds_wait<0>(kb[0], kb[1], kb[2], kb[3]);
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(i < 4 ? ka[i] : kb[i - 4], qf[0][i], acc, 0, 0, 0);
    }
    const float e0 = __builtin_amdgcn_exp2f(s[2 * i] * cs - mc);
    const float e1 = __builtin_amdgcn_exp2f(s[2 * i + 1] * cs - mc);
    packed[i] = pack_bf16(e0, e1);
    if (i & 1) sum1 = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, packed[i]), ones, sum1, false);
    else sum0 = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, packed[i]), ones, sum0, false);
    if (WITH_QK) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // one MFMA ...
      __builtin_amdgcn_sched_group_barrier(0x002, 2, 0);   // ... two fma,
      __builtin_amdgcn_sched_group_barrier(0x400, 2, 0);   // two exp2,
      __builtin_amdgcn_sched_group_barrier(0x002, 2, 0);   // the bf16 pack and the dot product with ones
    }
  }
  l_part += sum0 + sum1;
  if (WITH_QK) s_next = acc;
  uint4 w0 = {packed[0], packed[1], packed[2], packed[3]};
  uint4 w1 = {packed[4], packed[5], packed[6], packed[7]};
  pf0 = __builtin_bit_cast(bf16x8, w0);
  pf1 = __builtin_bit_cast(bf16x8, w1);
}

// O^T += V^T P^T with the P fragments already packed
__device__ __forceinline__ void pv_packed(unsigned vaddr, const LaneOffsets& lo, VFrags& vf0, const bf16x8& pf0,
                                          const bf16x8& pf1, f32x16 (&oacc)[1][4]) {
  VFrags vf1;
  v_fetch<1>(vaddr, lo, vf1);
  lds_wait<8>(vf0.f[0], vf0.f[1], vf0.f[2], vf0.f[3]);
#pragma unroll
  for (int dt = 0; dt < 4; ++dt) {
    if (dt == 0) mfma_acc<true>(oacc[0][dt], vf0.f[dt], pf0);
    else mfma_acc<false>(oacc[0][dt], vf0.f[dt], pf0);
  }
  lds_wait<0>(vf1.f[0], vf1.f[1], vf1.f[2], vf1.f[3]);
#pragma unroll
  for (int dt = 0; dt < 4; ++dt) {
    if (dt == 0) mfma_acc<true>(oacc[0][dt], vf1.f[dt], pf1);
    else mfma_acc<false>(oacc[0][dt], vf1.f[dt], pf1);
  }
}

template <int NT>
__device__ __forceinline__ void zero_state(f32x16 (&oacc)[NT][4], float (&m_ref)[NT], float (&l_part)[NT]) {
#pragma unroll
  for (int rt = 0; rt < NT; ++rt) {
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int v = 0; v < 16; ++v) oacc[rt][dt][v] = 0.f;
    m_ref[rt] = -INFINITY;
    l_part[rt] = 0.f;
  }
}

// ---- work units ---------------------------------------------------------------------------
// A unit is consumed in steps of 32 keys; step t covers keys [128 kv_begin + 32 t, +32), i.e. slice
// t % 4 of block kv_begin + t / 4, and every slice has the same layout in LDS.

struct UnitState {
  f32x16 oacc[1][4];
  float m_ref[1], l_part[1];
};

// Normalise and store the rows of a finished unit, or hand its un-normalised state to the merge pass.
__device__ __forceinline__ void finish_unit(const RunParams& p, const XyDevUnit& u, const XyDevSeq& sq,
                                            const UnitCtx& c, const Rows<1>& r, UnitState& st, int row_base,
                                            int col, int half) {
  mfma_results_ready(st.oacc[0][0], st.oacc[0][1], st.oacc[0][2], st.oacc[0][3]);
  const float l_tot = st.l_part[0] + other_half(st.l_part[0]);
  const float m2 = (st.m_ref[0] == -INFINITY) ? -INFINITY : st.m_ref[0] * p.c;     // running max, log2 units
  if (!r.valid[0]) return;
  const int rho = row_base + col;
  const int tl = rho / c.hc, hl = rho - tl * c.hc;
  if (u.ws_offset >= 0) {   // K/V-split unit
    float* w = p.ws + u.ws_offset;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int a = 0; a < 4; ++a) {
        f32x4 x = {st.oacc[0][dt][4 * a], st.oacc[0][dt][4 * a + 1], st.oacc[0][dt][4 * a + 2],
                   st.oacc[0][dt][4 * a + 3]};
        *reinterpret_cast<f32x4*>(w + (int64_t)rho * kD + 32 * dt + 8 * a + 4 * half) = x;
      }
    if (half == 0) {
      w[(int64_t)c.rows * kD + rho] = m2;
      w[(int64_t)c.rows * kD + c.rows + rho] = l_tot;
    }
  } else {
    const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
    uint16_t* o = p.out + (int64_t)(sq.token_start + u.q_begin + tl) * p.o_ts + (int64_t)(u.head_begin + hl) * p.o_hs;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int a = 0; a < 4; ++a) {
        uint2 w2;
        w2.x = pack_bf16(st.oacc[0][dt][4 * a] * inv, st.oacc[0][dt][4 * a + 1] * inv);
        w2.y = pack_bf16(st.oacc[0][dt][4 * a + 2] * inv, st.oacc[0][dt][4 * a + 3] * inv);
        *reinterpret_cast<uint2*>(o + 32 * dt + 8 * a + 4 * half) = w2;
      }
  }
}

// A unit with more than 32 rows (MFMA-bound): the eight wavefronts of the workgroup work together.
// Wavefront w owns rows [32w, 32w + 32) and sees every key; the block's K and V tiles are loaded
// cooperatively (wavefront w fetches rows [16w, 16w + 16)) and two block pairs are resident.
// Software pipeline: the QK^T MFMAs of step t + 1 are interleaved with the exponentials of step t,
// so the matrix pipe works while the vector ALU does the softmax (the paper's cube / vector overlap
// of section 4.2.1, inside one wavefront); the second wavefront of the SIMD fills what is left.
// Two barriers per block: "next block has landed" before its first QK^T, and "everybody is done
// with this block" before its tile pair is refilled.
__device__ __forceinline__ void process_wide(const RunParams& p, const XyDevUnit& u, const XyDevSeq& sq,
                                             unsigned char* smem, const LaneOffsets& lo, const DmaOffsets& dof) {
  constexpr int NT = 1;
  const int tid = threadIdx.x, lane = tid & 63, col = lane & 31, half = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);      // wavefront-uniform: branches on it stay scalar
  const UnitCtx c = make_ctx(p, u, sq);
  const int row_base = 32 * wave;
  const bool active = row_base < c.rows;
  Rows<NT> r;
  bf16x8 qf[NT][8];
  setup_rows<NT>(p, u, sq, c, row_base, col, half, r, qf);
  // smallest causal limit among this wavefront's rows (rows are token-major, so it is the first row's)
  const int mask_from = c.tree ? c.ctx : c.ctx + u.q_begin + row_base / c.hc + 1;
  UnitState st;
  zero_state<NT>(st.oacc, st.m_ref, st.l_part);

  const XY_CONST int32_t* table = as_const(p.block_table) + (int64_t)u.seq * p.max_blocks;
  const int last_page = (sq.ctx_len + sq.q_len - 1) >> p.page_shift;
  const int64_t head_off = (int64_t)c.kvh * p.kv_hs;
  const int nblk = u.kv_end - u.kv_begin;
  const int jfirst = u.kv_begin * kB;
  const int nsteps = (min(u.kv_end * kB, c.key_end) - jfirst + 31) >> 5;   // steps holding a visible key

  __syncthreads();            // the previous unit's readers are done with the tiles
  {                           // this wavefront's sixteen rows of the first tile
    const int64_t base = kv_row_offset(table, jfirst + 16 * wave, last_page, p) + head_off;
    load_rows_async<4>(p.k + base, p.v + base, p.kv_ts, 0, smem + wave * 4096,
                       smem + kTileBytes + wave * 4096, dof, true, true);
  }
  wait_vmcnt<0>();
  __syncthreads();

  // One step; s_cur holds S^T of step t (computed one step ahead), s_next receives that of step t + 1.
  auto step = [&](const int t, f32x16& s_cur, f32x16& s_next) {
    const int blk = t >> 2, slot = t & 3;
    const unsigned kaddr = lds_addr(smem + (blk & 1) * 2 * kTileBytes) + slot * 8192;
    if (slot == 0 && blk + 1 < nblk) {        // stream the next block into the other (free) tile pair
      unsigned char* nk = smem + ((blk + 1) & 1) * 2 * kTileBytes;
      const int64_t base = kv_row_offset(table, jfirst + kB * (blk + 1) + 16 * wave, last_page, p) + head_off;
      load_rows_async<4>(p.k + base, p.v + base, p.kv_ts, 0, nk + wave * 4096,
                         nk + kTileBytes + wave * 4096, dof, true, true);
    }
    const int tn = t + 1;
    const bool more = tn < nsteps;
    if (more && (tn & 3) == 0) {              // the next step opens a new block: its tiles must have landed
      wait_vmcnt<0>();
      __syncthreads();
    }
    if (active) {
      VFrags vf;
      const unsigned vaddr = kaddr + kTileBytes;
      v_fetch<0>(vaddr, lo, vf);              // the first V fragments arrive while the softmax runs
      const int j = jfirst + 32 * t;
      if (j + 32 > mask_from) {
        f32x16 sm[1] = {s_cur};
        mask_step<NT>(p, sq, c, r, j + 8 * half, sm);
        s_cur = sm[0];
      }
      const float mc = softmax_max(p.c, s_cur, st.m_ref[0], st.l_part[0], st.oacc);
      bf16x8 pf0, pf1;
      const unsigned kaddr_next = lds_addr(smem + ((tn >> 2) & 1) * 2 * kTileBytes) + (tn & 3) * 8192;
      if (more)
        exp_with_next_qk<true>(p.c, mc, s_cur, st.l_part[0], pf0, pf1, kaddr_next, lo, qf, s_next);
      else
        exp_with_next_qk<false>(p.c, mc, s_cur, st.l_part[0], pf0, pf1, kaddr_next, lo, qf, s_next);
      pv_packed(vaddr, lo, vf, pf0, pf1, st.oacc);
    }
    if (slot == 3 && more) __syncthreads();   // everybody is done with this block's tile pair
  };

  f32x16 sa, sb;
  if (active) {
    f32x16 first[1];
    qk_step<NT>(lds_addr(smem), lo, qf, first);
    sa = first[0];
  }
#pragma unroll 1
  for (int t = 0; t < nsteps; t += 2) {       // two steps per trip: the score tiles alternate without copies
    step(t, sa, sb);
    if (t + 1 < nsteps) step(t + 1, sb, sa);
  }
  finish_unit(p, u, sq, c, r, st, row_base, col, half);
}

// A unit with at most 32 rows (decode, short verify; bandwidth-bound): ONE wavefront processes the
// whole unit on its own, streaming 32-key slices through a private 16 KB ring (a K slot and a V slot,
// each refilled as soon as it has been consumed).  No barrier, no cross-wavefront merge: eight such
// units are in flight per CU and hide each other's latencies.
__device__ __forceinline__ void process_solo(const RunParams& p, const XyDevUnit& u, const XyDevSeq& sq,
                                             unsigned char* smem, const LaneOffsets& lo, const DmaOffsets& dof) {
  constexpr int NT = 1;
  const int tid = threadIdx.x, lane = tid & 63, col = lane & 31, half = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const UnitCtx c = make_ctx(p, u, sq);
  Rows<NT> r;
  bf16x8 qf[NT][8];
  setup_rows<NT>(p, u, sq, c, 0, col, half, r, qf);
  const int mask_from = c.tree ? c.ctx : c.ctx + u.q_begin + 1;
  UnitState st;
  zero_state<NT>(st.oacc, st.m_ref, st.l_part);

  const XY_CONST int32_t* table = as_const(p.block_table) + (int64_t)u.seq * p.max_blocks;
  const int last_page = (sq.ctx_len + sq.q_len - 1) >> p.page_shift;
  const int64_t head_off = (int64_t)c.kvh * p.kv_hs;
  const int jfirst = u.kv_begin * kB;
  const int nsteps = (min(u.kv_end * kB, c.key_end) - jfirst + 31) >> 5;
  unsigned char* ring = smem + wave * 16384;        // [K slot | V slot]
  const unsigned kaddr = lds_addr(ring), vaddr = kaddr + 8192;
  // a 32-key slice starting at key j: two runs of sixteen rows, each inside one page; eight
  // instructions per tensor, which is what the waits below count
  auto load_slice = [&](const int j, const bool want_k, const bool want_v) {
    const int64_t b0 = kv_row_offset(table, j, last_page, p) + head_off;
    const int64_t b1 = kv_row_offset(table, j + 16, last_page, p) + head_off;
    load_rows_async<4>(p.k + b0, p.v + b0, p.kv_ts, 0, ring, ring + 8192, dof, want_k, want_v);
    load_rows_async<4>(p.k + b1, p.v + b1, p.kv_ts, 0, ring + 4096, ring + 8192 + 4096, dof, want_k, want_v);
  };
  load_slice(jfirst, true, false);          // issue order K, V
  load_slice(jfirst, false, true);
#pragma unroll 1
  for (int t = 0; t < nsteps; ++t) {
    wait_vmcnt<8>();                          // K(t) has landed; only V(t) may still be in flight
    f32x16 s[NT];
    VFrags vf;
    qk_step<NT>(kaddr, lo, qf, s);            // all K reads have completed when this returns
    const int tn = t + 1;
    if (tn < nsteps) {        // K slot is free again: refill it with the next slice
      load_slice(jfirst + 32 * tn, true, false);
      wait_vmcnt<8>();        // V(t) has landed; the K refill stays in flight
    } else {
      wait_vmcnt<0>();
    }
    v_fetch<0>(vaddr, lo, vf);                // the first V fragments arrive while the softmax runs
    const int j = jfirst + 32 * t;
    if (j + 32 > mask_from) mask_step<NT>(p, sq, c, r, j + 8 * half, s);
    softmax_step<NT>(p.c, s, st.m_ref, st.l_part, st.oacc);
    pv_step<NT>(vaddr, lo, vf, s, st.oacc);   // all V reads have completed when this returns
    if (tn < nsteps) load_slice(jfirst + 32 * tn, false, true);
  }
  finish_unit(p, u, sq, c, r, st, 0, col, half);
}

// Every workgroup is one worker of the Task-Table (paper section 3.3).  It first works through the
// wide units of its list together, then its eight wavefronts draw the remaining (bandwidth-bound)
// units of the same list one by one from a shared cursor, each wavefront finishing whole units
// on its own.
__global__ __launch_bounds__(kThreads) void xy_attn_units_kernel(RunParams p) {
  __shared__ __attribute__((aligned(16))) unsigned char smem[4 * kTileBytes];
  __shared__ int cursor;
  // consecutive workgroup ids land on different XCDs; give each XCD a contiguous range of workers
  int worker = blockIdx.x;
  if ((p.num_workers & 7) == 0) worker = (blockIdx.x & 7) * (p.num_workers >> 3) + (blockIdx.x >> 3);
  const int begin = as_const(p.worker_offsets)[worker], end = as_const(p.worker_offsets)[worker + 1];
  const LaneOffsets lo = make_lane_offsets(threadIdx.x & 63);
  const DmaOffsets dof = make_dma_offsets(threadIdx.x & 63, p.kv_ts);
  if (threadIdx.x == 0) cursor = begin;
#pragma unroll 1
  for (int i = begin; i < end; ++i) {
    const XyDevUnit u = load_const(p.units + i);
    if (u.q_count * u.head_count <= 32) continue;
    const XyDevSeq sq = load_const(p.seqs + u.seq);
    process_wide(p, u, sq, smem, lo, dof);
  }
  __syncthreads();            // the tiles are free; the cursor is initialised
#pragma unroll 1
  while (true) {
    int got = 0;
    if ((threadIdx.x & 63) == 0) got = atomicAdd(&cursor, 1);
    const int i = __builtin_amdgcn_readfirstlane(got);
    if (i >= end) break;
    const XyDevUnit u = load_const(p.units + i);
    if (u.q_count * u.head_count > 32) continue;
    const XyDevSeq sq = load_const(p.seqs + u.seq);
    process_solo(p, u, sq, smem, lo, dof);
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

// Argument checks of a run (everything that can fail before device work is enqueued).
static int check_run_args(xy_attn_plan* plan, const void* q, int64_t q_ts, int64_t q_hs, const void* k_cache,
                          const void* v_cache, int64_t kv_bs, int64_t kv_hs, int64_t kv_ts,
                          const int32_t* block_table, const uint32_t* tree_masks, void* out, int64_t o_ts,
                          int64_t o_hs, void* workspace, size_t workspace_bytes, float softmax_scale) {
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
  if (int rc = check_run_args(plan, q, q_ts, q_hs, k_cache, v_cache, kv_bs, kv_hs, kv_ts, block_table, tree_masks,
                              out, o_ts, o_hs, workspace, workspace_bytes, softmax_scale))
    return rc;

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
  p.page_mask = plan->cfg.block_size - 1;
  p.page_shift = plan->cfg.block_size == 16 ? 4 : plan->cfg.block_size == 32 ? 5 : plan->cfg.block_size == 64 ? 6 : 7;
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

// ---- K/V append (section 4.1.1: the cache holds historical and newly generated tokens) --------
// One thread moves one 16-byte chunk: thread index = ((token * Hkv + kv head) * 2 + (K | V)) * 16 + chunk.
// The sixteen threads of a row read 256 contiguous bytes and write 256 contiguous bytes.  The owning
// sequence of a token is found by bisection over the packed start positions.
__global__ __launch_bounds__(256) void xy_attn_append_kernel(const XyDevSeq* __restrict__ seqs, int num_seqs,
                                                             int64_t total_tokens, int num_kv_heads,
                                                             const uint16_t* __restrict__ k_new,
                                                             const uint16_t* __restrict__ v_new, int64_t n_ts,
                                                             int64_t n_hs, uint16_t* __restrict__ k_cache,
                                                             uint16_t* __restrict__ v_cache, int64_t kv_bs,
                                                             int64_t kv_hs, int64_t kv_ts,
                                                             const int32_t* __restrict__ block_table,
                                                             int max_blocks, int page_shift) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int chunk = (int)(idx & 15), is_v = (int)((idx >> 4) & 1);
  const int64_t row = idx >> 5;                     // token * Hkv + kv head
  const int64_t t = row / num_kv_heads;
  const int g = (int)(row - t * num_kv_heads);
  if (t >= total_tokens) return;
  int lo = 0, hi = num_seqs - 1;                    // last sequence whose token_start <= t
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (seqs[mid].token_start <= t) lo = mid; else hi = mid - 1;
  }
  const XyDevSeq sq = seqs[lo];
  const int j = sq.ctx_len + (int)(t - sq.token_start);          // key position of this token
  const int64_t block = block_table[(int64_t)lo * max_blocks + (j >> page_shift)];
  const uint16_t* src = (is_v ? v_new : k_new) + t * n_ts + (int64_t)g * n_hs + chunk * 8;
  uint16_t* dst = (is_v ? v_cache : k_cache) + block * kv_bs + (int64_t)g * kv_hs + (int64_t)(j & ((1 << page_shift) - 1)) * kv_ts + chunk * 8;
  *reinterpret_cast<uint4*>(dst) = *reinterpret_cast<const uint4*>(src);
}

extern "C" int xy_attn_append_kv(xy_attn_plan* plan, const void* k_new, const void* v_new, int64_t n_ts,
                                 int64_t n_hs, void* k_cache, void* v_cache, int64_t kv_bs, int64_t kv_hs,
                                 int64_t kv_ts, const int32_t* block_table, void* hip_stream) {
  if (!plan) return XY_ERR_ARG;
  if (plan->total_tokens == 0) return XY_OK;
  if (!k_new || !v_new || !k_cache || !v_cache || !block_table) return XY_ERR_ARG;
  const int64_t strides[] = {n_ts, n_hs, kv_bs, kv_hs, kv_ts};
  for (int64_t s : strides)
    if (s < 0 || (s & 7)) return XY_ERR_ARG;
  if (n_hs < kD || kv_ts < kD) return XY_ERR_ARG;
  const uintptr_t ptrs[] = {(uintptr_t)k_new, (uintptr_t)v_new, (uintptr_t)k_cache, (uintptr_t)v_cache};
  for (uintptr_t a : ptrs)
    if (a & 15) return XY_ERR_ARG;
  if (int rc = xy_attn_plan_upload(plan)) return rc;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev != plan->device) return XY_ERR_ARG;
  const int64_t threads = plan->total_tokens * plan->cfg.num_kv_heads * 32;
  const unsigned blocks = (unsigned)((threads + 255) / 256);
  hipLaunchKernelGGL(xy_attn_append_kernel, dim3(blocks), dim3(256), 0, static_cast<hipStream_t>(hip_stream),
                     static_cast<const XyDevSeq*>(plan->d_seqs), plan->num_seqs, plan->total_tokens,
                     plan->cfg.num_kv_heads, static_cast<const uint16_t*>(k_new),
                     static_cast<const uint16_t*>(v_new), n_ts, n_hs, static_cast<uint16_t*>(k_cache),
                     static_cast<uint16_t*>(v_cache), kv_bs, kv_hs, kv_ts, block_table,
                     plan->cfg.max_blocks_per_seq,
                     plan->cfg.block_size == 16 ? 4 : plan->cfg.block_size == 32 ? 5 : plan->cfg.block_size == 64 ? 6 : 7);
  if (hipGetLastError() != hipSuccess) return XY_ERR_HIP;
  return XY_OK;
}

// ---- copy-on-write of partly reused blocks (section 4.1.1) ------------------------------------
struct CopyBatch {
  xy_kv_copy c[32];
};

// Workgroup (copy, KV head, K | V) moves rows x 256 bytes in 16-byte chunks.
__global__ __launch_bounds__(256) void xy_attn_copy_rows_kernel(CopyBatch batch, int num_kv_heads,
                                                                uint16_t* __restrict__ k_cache,
                                                                uint16_t* __restrict__ v_cache, int64_t kv_bs,
                                                                int64_t kv_hs, int64_t kv_ts) {
  const int is_v = blockIdx.x & 1;
  const int g = (blockIdx.x >> 1) % num_kv_heads;
  const xy_kv_copy cp = batch.c[(blockIdx.x >> 1) / num_kv_heads];
  uint16_t* cache = is_v ? v_cache : k_cache;
  const uint16_t* src = cache + (int64_t)cp.src_block * kv_bs + (int64_t)g * kv_hs;
  uint16_t* dst = cache + (int64_t)cp.dst_block * kv_bs + (int64_t)g * kv_hs;
  for (int i = threadIdx.x; i < cp.rows * 16; i += blockDim.x) {
    const int64_t off = (int64_t)(i >> 4) * kv_ts + (i & 15) * 8;
    *reinterpret_cast<uint4*>(dst + off) = *reinterpret_cast<const uint4*>(src + off);
  }
}

extern "C" int xy_attn_copy_block_rows(const xy_kv_copy* copies, int32_t n, int32_t num_kv_heads, void* k_cache,
                                       void* v_cache, int64_t kv_bs, int64_t kv_hs, int64_t kv_ts,
                                       void* hip_stream) {
  if (n < 0 || num_kv_heads < 1) return XY_ERR_ARG;
  if (n == 0) return XY_OK;
  if (!copies || !k_cache || !v_cache) return XY_ERR_ARG;
  const int64_t strides[] = {kv_bs, kv_hs, kv_ts};
  for (int64_t st : strides)
    if (st < 0 || (st & 7)) return XY_ERR_ARG;
  if (kv_ts < kD || ((uintptr_t)k_cache & 15) || ((uintptr_t)v_cache & 15)) return XY_ERR_ARG;
  for (int32_t i = 0; i < n; ++i)
    if (copies[i].rows < 0 || copies[i].src_block < 0 || copies[i].dst_block < 0) return XY_ERR_ARG;
  for (int32_t first = 0; first < n; first += 32) {
    CopyBatch batch;
    const int32_t cnt = std::min(32, n - first);
    for (int32_t i = 0; i < cnt; ++i) batch.c[i] = copies[first + i];
    hipLaunchKernelGGL(xy_attn_copy_rows_kernel, dim3((unsigned)(cnt * num_kv_heads * 2)), dim3(256), 0,
                       static_cast<hipStream_t>(hip_stream), batch, num_kv_heads, static_cast<uint16_t*>(k_cache),
                       static_cast<uint16_t*>(v_cache), kv_bs, kv_hs, kv_ts);
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

extern "C" int xy_attn_run_fused_qkv(xy_attn_plan* plan, const void* qkv, int64_t qkv_ts, int64_t qkv_hs,
                                     void* k_cache, void* v_cache, int64_t kv_bs, int64_t kv_hs, int64_t kv_ts,
                                     const int32_t* block_table, const uint32_t* tree_masks, void* out,
                                     int64_t o_ts, int64_t o_hs, void* workspace, size_t workspace_bytes,
                                     float softmax_scale, void* hip_stream) {
  if (!plan) return XY_ERR_ARG;
  if (plan->units.empty()) return XY_OK;
  if (!qkv || qkv_hs < kD || (qkv_hs & 7)) return XY_ERR_ARG;
  const uint16_t* base = static_cast<const uint16_t*>(qkv);
  const uint16_t* k_new = base + (int64_t)plan->cfg.num_q_heads * qkv_hs;
  const uint16_t* v_new = k_new + (int64_t)plan->cfg.num_kv_heads * qkv_hs;
  // validate the attention arguments first: a call that fails enqueues no device work
  if (int rc = check_run_args(plan, qkv, qkv_ts, qkv_hs, k_cache, v_cache, kv_bs, kv_hs, kv_ts, block_table,
                              tree_masks, out, o_ts, o_hs, workspace, workspace_bytes, softmax_scale))
    return rc;
  if (int rc = xy_attn_append_kv(plan, k_new, v_new, qkv_ts, qkv_hs, k_cache, v_cache, kv_bs, kv_hs, kv_ts,
                                 block_table, hip_stream))
    return rc;
  return run_impl(XY_PHASE_UNITS | XY_PHASE_MERGE, plan, qkv, qkv_ts, qkv_hs, k_cache, v_cache, kv_bs, kv_hs,
                  kv_ts, block_table, tree_masks, out, o_ts, o_hs, workspace, workspace_bytes, softmax_scale,
                  hip_stream);
}
