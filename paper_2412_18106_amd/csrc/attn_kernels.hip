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
//  * 256 threads = 4 wavefronts per workgroup, one per SIMD (so each may use all 512
//    registers of its SIMD lane), one workgroup per CU, 128 KB LDS; K and V stream from
//    HBM straight into LDS (no staging registers) while earlier blocks are consumed.
//  * Scores are produced transposed, S^T = K Q^T, with the 32x32x16 bf16 MFMA:
//    a lane then owns ONE query row (max / sum need one cross-lane exchange), the
//    accumulator registers of S^T are already the B operand of O^T += V^T P^T,
//    and rescaling O^T is one scalar per lane.
//  * V^T fragments come from the row-major V tile in LDS through the
//    transposing LDS read (ds_read_b64_tr_b16).
//  * rows = tokens x heads of one KV head (GQA sharing): a unit with more than
//    32 rows gives each wavefront 64 rows and every key, the wavefronts sharing
//    the K/V stream (every fragment read from LDS feeds two MFMAs); a unit with
//    up to 32 rows (decode, short verify) is processed by a single wavefront
//    streaming 32-key slices through a private LDS ring, so a CU has four such
//    units in flight and no barrier between them.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <mutex>

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
constexpr int kThreads = 256;        // 4 wavefronts: one per SIMD
constexpr float kPrescaleMaxC = 0.25f;    // largest c = scale * log2(e) that is folded into Q (wide units)
// Dynamic assignment: the cursor of the shared list, kDoneGroups counts of finished workgroups and the
// count of finished groups, kCounterStride ints (one 128-byte line) apart.
constexpr int kDoneGroups = 8;
constexpr int kCounterStride = 32;
constexpr float kLazyRescale = 8.0f;      // log2 units the running max may lag behind
// Placement of the vector work of a wide iteration between its MFMAs: how many of the 32 exponentials, 16 bf16
// packings and 32 row-sum additions are done before each of the 32 gaps (made by gap_tables.py of this package
// from measured issue costs; a unit test compares them with what that module prints).
#define XY_GAP_TABLE_EXP {0, 2, 4, 5, 6, 7, 8, 10, 11, 12, 13, 14, 14, 15, 16, 17, 18, 19, 21, 22, 22, 22, 24, 25, 26, 27, 28, 30, 30, 31, 32, 32, 32}
#define XY_GAP_TABLE_CVT {0, 0, 0, 1, 1, 2, 3, 3, 3, 4, 5, 5, 5, 6, 7, 7, 8, 8, 8, 9, 9, 10, 10, 10, 11, 12, 13, 13, 13, 14, 15, 16, 16}
#define XY_GAP_TABLE_ADD {0, 0, 1, 2, 2, 3, 5, 5, 7, 7, 9, 10, 11, 11, 13, 14, 15, 16, 17, 17, 18, 19, 20, 21, 22, 23, 25, 25, 26, 27, 29, 32, 32}
constexpr float kRowSumLimit = 18446744073709551616.f;      // 2^64: a wide unit whose row sums stay below was computed without overflow

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
  int32_t num_units;                 // all units, the shared list of XY_ASSIGN_DYNAMIC included
  int32_t* counters;                 // plan with a shared list: its cursor and the finished-workgroup counts (kCounterStride apart); else null
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

// Cache policy of the K/V loads of the narrow (bandwidth-bound) units: every byte is read once per launch, so the
// loads carry the non-temporal hint and leave the L2 to data that is used again (measured: decode-heavy steps
// 9-11 % faster, 5.4 -> 5.9 TB/s).  The wide units leave it off: their K/V is shared by the tiles of a sequence
// that run side by side on a chiplet.
constexpr int kReadOnce = 2;      // the nt bit of the instruction's cache-policy field

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
          (__attribute__((address_space(3))) void*)(lds_k + e * 1024), 16, 0, kReadOnce);
    if (want_v)
      __builtin_amdgcn_global_load_lds(
          (const __attribute__((address_space(1))) void*)(reinterpret_cast<const char*>(vg + rows) + (size_t)dof.v),
          (__attribute__((address_space(3))) void*)(lds_v + e * 1024), 16, 0, kReadOnce);
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

// Rows [first_row, 32) of a 32-row V slice in LDS are set to zero.  The last step of a unit may cover slots behind
// the unit's last key (the rest of a page, keys of later rows): their probabilities are exactly zero, but 0 x NaN
// and 0 x Inf are not, and a cache that was never initialised may hold such patterns there.  K needs nothing of
// the kind: a masked score is overwritten, not multiplied.  Every wavefront that reads the slice clears the same
// rows itself before it reads (the writes are idempotent), so no barrier is needed.
__device__ __forceinline__ void zero_tail_rows(unsigned slice_addr, int first_row, int lane) {
  // two registers in all (the units that need this are at their register limit): one address, one zero
  unsigned addr = slice_addr + (unsigned)(first_row + (lane >> 4)) * 256u + (unsigned)(lane & 15) * 16u;
  const unsigned zero = 0u;
  for (int r = first_row + (lane >> 4); r < 32; r += 4) {
    asm volatile("ds_write_b32 %0, %1 offset:0\n\tds_write_b32 %0, %1 offset:4\n\t"
                 "ds_write_b32 %0, %1 offset:8\n\tds_write_b32 %0, %1 offset:12"
                 :: "v"(addr), "v"(zero) : "memory");
    addr += 1024u;
  }
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");     // before the hand-issued fragment reads that follow
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
      // only the rows that asked move their reference: a row's arithmetic does not depend on its neighbours' keys
      const float m_new = bump ? fmaxf(m_ref[rt], mx) : m_ref[rt];
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

// ---- wide units (more than 32 rows, MFMA-bound) -------------------------------------------------------
// One wavefront per SIMD, 64 rows (two 32-row tiles) per wavefront: every K or V fragment read from LDS
// feeds two MFMAs, which halves the LDS read traffic per MFMA against one tile per wavefront.  The price is
// registers: the O^T accumulators (2 x 4 x 16) and the Q fragments (2 x 8 x 4) live in AGPRs, S^T, P and the
// K / V fragments in VGPRs, about 450 of the 512 a lone wavefront may use.  With nobody else on the SIMD
// there is nothing to hide a stall behind, so the MFMAs and the LDS reads are issued by hand in a fixed
// interleave, every wait is for exactly the fragment that is needed next, and the compiler's output is
// checked at build time for what it cannot know about such instructions (no spills, no use of a result
// or an operand inside the wait states the hardware needs).

template <int T>      // one 32-wide d tile of v_fetch
__device__ __forceinline__ void v_fetch_one(unsigned vaddr, const LaneOffsets& lo, int dt, bf16x8& f) {
  const unsigned a = vaddr + lo.v[dt];
  const s16x4 r0 = lds_read_tr16_b64<T * 16 * 256>(a);
  const s16x4 r1 = lds_read_tr16_b64<T * 16 * 256 + 4 * 256>(a);
  s16x8 w;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    w[e] = r0[e];
    w[4 + e] = r1[e];
  }
  f = __builtin_bit_cast(bf16x8, w);
}

// O^T tile += V^T fragment x P fragment, accumulator in AGPRs
__device__ __forceinline__ void mfma_pv(f32x16& acc, const bf16x8& vfrag, const bf16x8& pfrag) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(acc) : "v"(vfrag), "v"(pfrag));
}
// wait states between a vector-ALU write of an MFMA operand and a hand-issued MFMA
__device__ __forceinline__ void valu_to_mfma_gap() { asm volatile("s_nop 4"); }
// The compiler does not know that the registers written by a hand-issued MFMA are not valid yet: where
// control flow merges it may copy them right behind the MFMA.  These statements sit directly behind the
// last MFMA of a sequence (volatile keeps the order, the operands keep every use of the results
// behind them) and pad the wait states a vector-ALU access of an MFMA result needs: settle covers a copy
// the compiler may place there, ready covers a read of the values.
__device__ __forceinline__ void mfma_settle(f32x16& a) { asm volatile("s_nop 7\n\ts_nop 4" : "+v"(a)); }
__device__ __forceinline__ void settle_a(f32x16& a, f32x16& b, f32x16& c, f32x16& d) {
  asm volatile("s_nop 7\n\ts_nop 4" : "+a"(a), "+a"(b), "+a"(c), "+a"(d));
}
__device__ __forceinline__ void ready_a(f32x16& a, f32x16& b, f32x16& c, f32x16& d) {
  asm volatile("s_nop 7\n\ts_nop 7\n\ts_nop 7" : "+a"(a), "+a"(b), "+a"(c), "+a"(d));
}

template <int N>      // wait until at most N LDS requests are outstanding; tied to the fragment it protects
__device__ __forceinline__ void lds_wait1(bf16x8& a) {
  asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(a) : "n"(N) : "memory");
}

template <int N>      // the same for the two fragments of a pair of chunks
__device__ __forceinline__ void lds_wait2(bf16x8& a, bf16x8& b) {
  asm volatile("s_waitcnt lgkmcnt(%2)" : "+v"(a), "+v"(b) : "n"(N) : "memory");
}

__device__ __forceinline__ float max3(float a, float b, float c) { return fmaxf(fmaxf(a, b), c); }
// the same as one instruction on values that are known to be numbers (MFMA results: the compiler would first
// quiet each of them with a v_max of its own)
__device__ __forceinline__ float max3_raw(float a, float b, float c) {
  float r;
  asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
  return r;
}

// acc *= alpha without the accumulator leaving the AGPR file for good: the product is forced back into
// an AGPR tuple here, in the rare branch, so the loop-carried value keeps one register class and the
// pipelined path sees no copies.
__device__ __forceinline__ void scale_acc(f32x16& acc, const float alpha) {
  f32x16 t = acc * alpha;
  asm volatile("; rescaled accumulator back in the AGPR file" : "+a"(t));
  acc = t;
}

// A unit with more than 32 rows.  Wavefront w owns rows [64w, 64w + 64) as two 32-row tiles and sees every
// key.  K and V stream through a ring of four 64-key half blocks (32 KB each: 16 KB of K, 16 KB of V);
// a "step" is 32 keys, a "trip" two steps = one half block.
// Iteration t works on three steps at once (the paper's cube / vector overlap of section 4.2.1, at
// instruction level inside one wavefront): the QK^T MFMAs of step t + 1, the softmax arithmetic of step t
// and the PV MFMAs of step t - 1, as sixteen chunks of two MFMAs (one per row tile, sharing the chunk's
// K or V fragment) with a few vector instructions and one LDS request behind each MFMA.
// PRESCALE: Q carries the factor c = scale x log2(e), see the softmax notes inside.
template <bool PRESCALE, bool ROWS_CONTIGUOUS>
// force: the second pass over a unit whose optimistic pass overflowed (exact prefix in every iteration).  Returns
// whether the unit has to be run again that way (only when force is false; nothing has been written then).
__device__ __forceinline__ bool process_wide(const RunParams& p, const XyDevUnit& u, const XyDevSeq& sq,
                                             unsigned char* smem, int* overflow_flags, const bool force,
                                             const LaneOffsets& lo, const DmaOffsets& dof) {
  constexpr int NT = 2;
  const int tid = threadIdx.x, lane = tid & 63, col = lane & 31, half = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const UnitCtx c = make_ctx(p, u, sq);
  const int row_base = 64 * wave;
  const bool active = row_base < c.rows;
  Rows<NT> r;
  bf16x8 qf[NT][8];
  setup_rows<NT>(p, u, sq, c, row_base, col, half, r, qf);
  const int mask_from = c.tree ? c.ctx : c.ctx + u.q_begin + row_base / c.hc + 1;
  f32x16 oacc[NT][4];
  float m_ref[NT], l_part[NT][4];      // four running partial row sums per tile, added to in place (plain additions:
                                        // the bf16 dot-product instruction would hold the matrix pipe for 16 cycles)

  const XY_CONST int32_t* table = as_const(p.block_table) + (int64_t)u.seq * p.max_blocks;
  const int last_page = (sq.ctx_len + sq.q_len - 1) >> p.page_shift;
  const int64_t head_off = (int64_t)c.kvh * p.kv_hs;
  const int jfirst = u.kv_begin * kB;
  const int nsteps = (min(u.kv_end * kB, c.key_end) - jfirst + 31) >> 5;
  const float cs = p.c;

  // ---- softmax with the reference folded into the MFMA ------------------------------------------------
  // The wavefront is bound by the number of instructions it can issue, so the common path of the softmax
  // is cut to exp2, pack and row sum.  The first QK^T MFMA of a step starts from -m_ref (the row's running
  // reference, one value per lane, kept in sixteen registers) instead of zero, so S^T arrives already
  // relative to the reference; with PRESCALE, Q is pre-multiplied by c and S^T is the exponent itself.
  // No row maximum is taken on the common path, and none is looked for either: a row gets its reference from
  // the exact prefix below on the first step in which it sees a key (the true maximum of that step), and keeps
  // it.  Floating point does not care how far later scores lie above the reference as long as nothing
  // overflows - the probabilities, the row sums and the accumulators all carry the same power of two, which
  // the final division removes - so the unit is run optimistically and checked once, at its end: if a row
  // sum has left the range [0, 2^64) (an exponent beyond 2^127 makes it infinite, a mix of infinities NaN),
  // the whole unit is run again (the caller's next turn) with the exact prefix in every iteration, which keeps every probability
  // below 2^8 as the lazy rescale of the narrow path does.  That takes a score 64 log2 units (44 nats) above
  // the largest score of the row's first step: inputs made for it (the needle tests), not attention scores.
  // S^T is kept in "score units": log2 units when Q carries the factor c, raw q.k otherwise.
  const float u2l = PRESCALE ? 1.f : cs;                                   // score units -> log2 units
  const float lazy = PRESCALE ? kLazyRescale : kLazyRescale / cs;         // the lazy-rescale margin in score units
#pragma unroll
  for (int rt = 0; rt < NT; ++rt)
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      if (!PRESCALE) break;
      uint4 w = __builtin_bit_cast(uint4, qf[rt][ks]);
      unsigned* wp = reinterpret_cast<unsigned*>(&w);
#pragma unroll
      for (int i = 0; i < 4; ++i)
        wp[i] = pack_bf16(__uint_as_float(wp[i] << 16) * cs, __uint_as_float(wp[i] & 0xffff0000u) * cs);
      qf[rt][ks] = __builtin_bit_cast(bf16x8, w);
      asm volatile("; scaled Q fragment lives in the AGPR file from here on" : "+a"(qf[rt][ks]));
    }

#pragma unroll
  for (int rt = 0; rt < NT; ++rt) {
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int v = 0; v < 16; ++v) oacc[rt][dt][v] = 0.f;
    m_ref[rt] = -INFINITY;
#pragma unroll
    for (int i = 0; i < 4; ++i) l_part[rt][i] = 0.f;
  }
  // ---- the K/V stream (paged cache of section 4.1.1) ---------------------------------------------------
  // Half block h lives in ring slot h & 3; wavefronts 0-1 fetch 32 rows of K each, wavefronts 2-3 32 rows
  // of V.  A wavefront has nobody to hide behind on its SIMD, so the page-table entries of a request are
  // read (scalar loads) a whole trip before the request is set up, and K and V take the same
  // straight-line path (base pointer and swizzle offsets selected once per unit).
  const uint16_t* kv_base = (wave < 2 ? p.k : p.v) + head_off;
  unsigned dsel[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) dsel[e] = wave < 2 ? dof.k[e] : dof.v;
  const int row_sel = 32 * (wave & 1);
  auto page_entry = [&](const int h, const int g) -> int {      // h counts K half blocks for wavefronts 0-1, V for 2-3
    const int j = jfirst + 64 * h + row_sel + 16 * g;
    return table[min(j >> p.page_shift, last_page)];            // rows past the last page are redirected to it
  };
  auto request_half_block = [&](const int h, const int entry0, const int entry1) {
    unsigned char* dst = smem + (h & 3) * 32768 + (wave >> 1) * 16384 + (wave & 1) * 8192;
#pragma unroll
    for (int g = 0; g < 2; ++g) {      // sixteen rows share a page
      const int j = jfirst + 64 * h + row_sel + 16 * g;
      const uint16_t* src = kv_base + (int64_t)(g ? entry1 : entry0) * p.kv_bs + (int64_t)(j & p.page_mask) * p.kv_ts;
#pragma unroll
      for (int e = 0; e < 4; ++e)
        __builtin_amdgcn_global_load_lds(
            (const __attribute__((address_space(1))) void*)(reinterpret_cast<const char*>(src + (int64_t)(4 * e) * p.kv_ts) + (size_t)dsel[e]),
            (__attribute__((address_space(3))) void*)(dst + 4096 * g + 1024 * e), 16, 0, 0);
    }
  };
  // After the first four half blocks, the eight loads of a request are issued one by one during the trip
  // that follows its set-up, so that their data reaches LDS a kilobyte at a time, between the fragment
  // reads, instead of as one burst.
  // Where the two sixteen-row runs of a request come from (page-table entry, page stride, row in the page) is 64-bit
  // arithmetic on scalars, some thirty scalar instructions per trip, which a lone wavefront can hide behind nothing.
  // The lanes work the addresses out instead, 64 half blocks at a time - lane l holds those of half block
  // 64 * window + l - and a trip reads its four words out of that table.
  const uint16_t* rsrc0 = kv_base;
  const uint16_t* rsrc1 = kv_base;
  unsigned char* rdst = smem;
  unsigned src_lo[2] = {0u, 0u}, src_hi[2] = {0u, 0u};
  int window = -1;
  auto fill_table = [&](const int w) {
#pragma unroll
    for (int g = 0; g < 2; ++g) {
      // (64-bit: lanes far behind the unit's last half block look past any sequence length; they are clamped to
      // the last page like every row behind the sequence's end)
      const int64_t jl = (int64_t)jfirst + 64 * (64 * (int64_t)w + lane) + row_sel + 16 * g;
      const int page = (int)min(jl >> p.page_shift, (int64_t)last_page);
      const int entry = p.block_table[(int64_t)u.seq * p.max_blocks + page];
      const uint64_t a = (uint64_t)(kv_base + (int64_t)entry * p.kv_bs + (jl & p.page_mask) * p.kv_ts);
      src_lo[g] = (unsigned)a;
      src_hi[g] = (unsigned)(a >> 32);
    }
  };
  auto setup_request = [&](const int h) {
    rdst = smem + (h & 3) * 32768 + (wave >> 1) * 16384 + (wave & 1) * 8192;
    if ((h >> 6) != window) {         // once per 64 trips
      window = h >> 6;
      fill_table(window);
    }
    const int l = h & 63;
    // (the lane read returns a signed int: widened through unsigned, or a low word with its top bit set would
    // smear over the high word)
    rsrc0 = reinterpret_cast<const uint16_t*>(((uint64_t)(unsigned)__builtin_amdgcn_readlane((int)src_hi[0], l) << 32) |
                                              (uint64_t)(unsigned)__builtin_amdgcn_readlane((int)src_lo[0], l));
    rsrc1 = reinterpret_cast<const uint16_t*>(((uint64_t)(unsigned)__builtin_amdgcn_readlane((int)src_hi[1], l) << 32) |
                                              (uint64_t)(unsigned)__builtin_amdgcn_readlane((int)src_lo[1], l));
  };
  auto issue = [&](const int idx) {
    const int g = idx >> 2, e = idx & 3;
    const uint16_t* src = g ? rsrc1 : rsrc0;
    if (ROWS_CONTIGUOUS) {
      // rows of 256 bytes back to back: four rows further is 1 KB further in the cache and in LDS alike, so the
      // instruction's offset field moves both and the four loads of a page share their scalar operands
      asm volatile("" : "+v"(dsel[e]));      // keeps it a 32-bit lane offset on a scalar base, not a 64-bit address per lane
      const __attribute__((address_space(1))) void* from =
          (const __attribute__((address_space(1))) void*)(reinterpret_cast<const char*>(src) + (size_t)dsel[e]);
      __attribute__((address_space(3))) void* to = (__attribute__((address_space(3))) void*)(rdst + 4096 * g);
      switch (e) {      // the offset field is part of the instruction
        case 0: __builtin_amdgcn_global_load_lds(from, to, 16, 0, 0); break;
        case 1: __builtin_amdgcn_global_load_lds(from, to, 16, 1024, 0); break;
        case 2: __builtin_amdgcn_global_load_lds(from, to, 16, 2048, 0); break;
        default: __builtin_amdgcn_global_load_lds(from, to, 16, 3072, 0); break;
      }
    } else {
      __builtin_amdgcn_global_load_lds(
          (const __attribute__((address_space(1))) void*)(reinterpret_cast<const char*>(src + (int64_t)(4 * e) * p.kv_ts) + (size_t)dsel[e]),
          (__attribute__((address_space(3))) void*)(rdst + 4096 * g + 1024 * e), 16, 0, 0);
    }
  };
  auto k_slice = [&](const int t) { return lds_addr(smem) + ((t >> 1) & 3) * 32768 + (t & 1) * 8192; };

  __syncthreads();
#pragma unroll
  for (int h = 0; h < 4; ++h)
    if (h < 3 || wave < 2) request_half_block(h, page_entry(h, 0), page_entry(h, 1));      // K(0..3), V(0..2)
  wait_vmcnt<0>();
  __syncthreads();

  f32x16 sa[NT], sb[NT];
  bf16x8 pa[NT][2], pb[NT][2];
  bf16x8 kf[8], vf[8];
  f32x16 negm[NT];          // -m_ref of the lane's row in all sixteen registers (0 while the row has no reference)
#pragma unroll
  for (int rt = 0; rt < NT; ++rt)
#pragma unroll
    for (int v = 0; v < 16; ++v) negm[rt][v] = 0.f;
#pragma unroll
  for (int rt = 0; rt < NT; ++rt) asm volatile("" : "+v"(negm[rt]));

  auto request_k = [&](const unsigned kaddr, const int i) { kf[i] = lds_read_b128<0>(kaddr + lo.k[i]); };
  auto request_v = [&](const unsigned vaddr, const int i) {
    if (i < 4) v_fetch_one<0>(vaddr, lo, i, vf[i]);
    else v_fetch_one<1>(vaddr, lo, i - 4, vf[i]);
  };
  auto mfma_qk = [&](const int i, f32x16& s, const int rt) {     // chunk i of S^T(rt) = -m_ref + K Q^T
    if (i == 0)
      asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %3" : "=&v"(s) : "v"(kf[0]), "a"(qf[rt][0]), "v"(negm[rt]));
    else
      asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(s) : "v"(kf[i]), "a"(qf[rt][i]));
  };
  auto lane_max = [&](const f32x16& s) {
    const float a0 = max3(s[0], s[1], s[2]), a1 = max3(s[3], s[4], s[5]), a2 = max3(s[6], s[7], s[8]);
    const float a3 = max3(s[9], s[10], s[11]), a4 = max3(s[12], s[13], s[14]);
    return fmaxf(max3(a0, a1, a2), max3(a3, a4, s[15]));
  };
  // whether some valid row of this wavefront has no reference yet (it has not seen a key so far): the next
  // iteration then starts with the exact prefix too.  Wavefront-uniform; changes only where the references change.
  bool pending = true;

  // Exact prefix of an iteration (always in iteration 0, where it gives every row that sees a key its first
  // reference; after that only while some row is still waiting for its first key, or in the second pass over
  // a unit): the true row maximum of the masked s_in moves the reference, and everything
  // that was built against the old one follows it (the scores of this step, the row sums, the
  // accumulators, the packed probabilities of the previous step whose PV product is still to come), so
  // that the pipelined iteration runs unchanged afterwards.  A row that has a reference moves it by a
  // whole number of log2 units, which makes the factor a power of two: the packed probabilities are
  // rescaled without rounding.
  auto exact_prefix = [&](f32x16 (&s_in)[NT], bf16x8 (&p_in)[NT][2]) {
    ready_a(oacc[0][0], oacc[0][1], oacc[0][2], oacc[0][3]);
    ready_a(oacc[1][0], oacc[1][1], oacc[1][2], oacc[1][3]);
#pragma unroll
    for (int rt = 0; rt < NT; ++rt) {
      const float mx = max_both_halves(lane_max(s_in[rt]));       // relative to the reference
      const bool set = m_ref[rt] != -INFINITY;
      float delta, alpha;
      if (set) {
        const float d2 = mx >= lazy ? ceilf(mx * u2l) : 0.f;      // whole number of log2 units
        delta = PRESCALE ? d2 : d2 / cs;
        alpha = __builtin_amdgcn_exp2f(-d2);
        m_ref[rt] += delta;
      } else {
        delta = mx != -INFINITY ? mx : 0.f;
        alpha = 1.f;
        if (mx != -INFINITY) m_ref[rt] = mx;
      }
#pragma unroll
      for (int v = 0; v < 16; ++v) s_in[rt][v] -= delta;
#pragma unroll
      for (int i = 0; i < 4; ++i) l_part[rt][i] *= alpha;
#pragma unroll
      for (int dt = 0; dt < 4; ++dt) scale_acc(oacc[rt][dt], alpha);
#pragma unroll
      for (int h2 = 0; h2 < 2; ++h2) {
        uint4 w = __builtin_bit_cast(uint4, p_in[rt][h2]);
        unsigned* wp = reinterpret_cast<unsigned*>(&w);
#pragma unroll
        for (int i = 0; i < 4; ++i)
          wp[i] = pack_bf16(__uint_as_float(wp[i] << 16) * alpha, __uint_as_float(wp[i] & 0xffff0000u) * alpha);
        p_in[rt][h2] = __builtin_bit_cast(bf16x8, w);
      }
      const float nm = m_ref[rt] == -INFINITY ? 0.f : -m_ref[rt];
#pragma unroll
      for (int v = 0; v < 16; ++v) negm[rt][v] = nm;
      asm volatile("" : "+v"(negm[rt]));      // sixteen real registers from here on, nothing rebuilt next to the MFMA
    }
    pending = __builtin_amdgcn_ballot_w64((r.valid[0] && m_ref[0] == -INFINITY) || (r.valid[1] && m_ref[1] == -INFINITY)) != 0;
  };

  // Iteration t: QK^T of step t + 1 (chunks 0-7), exp2 / pack / row sum of step t (one pair of scores per
  // chunk), PV of step t - 1 (chunks 8-15).  The LDS request issued in a chunk is the fragment needed four
  // chunks later; par >= 0 numbers the iteration inside its trip for the K/V loads it issues.  Returns
  // whether the next iteration starts with the exact prefix; par == -2 marks the iteration after which no
  // other follows (its look-ahead scores are never read).
  // kaddr, vaddr, knext: LDS addresses of K of step t + 1, V of step t - 1 and K of step t + 2 (worked out
  // once per trip by the caller).
  auto iterate = [&](const bool exact, const int par, const int t, const unsigned kaddr, const unsigned vaddr,
                     const unsigned knext, f32x16 (&s_in)[NT], f32x16 (&s_out)[NT], bf16x8 (&p_in)[NT][2],
                     bf16x8 (&p_out)[NT][2]) -> bool {
    {
      const int j = jfirst + 32 * t;
      if (j + 32 > mask_from) mask_step<NT>(p, sq, c, r, j + 8 * half, s_in);
    }
    if (exact) {
      exact_prefix(s_in, p_in);
      valu_to_mfma_gap();       // the prefix rewrote the reference registers the first MFMA reads
    }
    lds_wait<0>(kf[0], kf[1], kf[2], kf[3]);
    unsigned packed[16];
    float e[32];
    // A lone wavefront issues in order: an MFMA that finds the matrix pipe busy holds up everything behind
    // it, and a gap with more than about 26 cycles of other instructions leaves the pipe idle.  So the
    // vector work of the iteration is dealt out over the 32 gaps behind its MFMAs (two per chunk) by a table
    // made offline from the issue costs measured for a lone wavefront (exp2 8.5 cycles, other vector
    // instructions 5, an LDS request 5.7, a scalar instruction 8.5, a wait 4.7), next to what a gap holds
    // anyway (LDS requests, waits, the K/V loads): about 24 cycles in every gap.  Scheduling barriers keep the
    // compiler from moving work between gaps.  The tables count, gap by gap, how many of the 32 exponentials,
    // 16 packings and 32 row-sum additions are done before that gap.
    constexpr int kExp[33] = XY_GAP_TABLE_EXP;
    constexpr int kCvt[33] = XY_GAP_TABLE_CVT;
    constexpr int kAdd[33] = XY_GAP_TABLE_ADD;
    auto exp_one = [&](const int j) {          // score j & 15 of row tile j >> 4
      e[j] = __builtin_amdgcn_exp2f(PRESCALE ? s_in[j >> 4][j & 15] : s_in[j >> 4][j & 15] * cs);
    };
    auto cvt_one = [&](const int g) {
      packed[g] = pack_bf16(e[2 * g], e[2 * g + 1]);
      asm volatile("" : "+v"(packed[g]));       // stays in this gap
    };
    auto add_one = [&](const int j) {
      l_part[j >> 4][j & 3] += e[j];
      asm volatile("" : "+v"(l_part[j >> 4][j & 3]));
    };
    auto gap_work = [&](const int k) {
#pragma unroll
      for (int j = kExp[k]; j < kExp[k + 1]; ++j) exp_one(j);
#pragma unroll
      for (int g = kCvt[k]; g < kCvt[k + 1]; ++g) cvt_one(g);
#pragma unroll
      for (int j = kAdd[k]; j < kAdd[k + 1]; ++j) add_one(j);
    };
#pragma unroll
    for (int ch = 0; ch < 16; ++ch) {
      // one wait per pair of chunks: before an even chunk, for its own fragment and the next one.  The
      // number allowed to stay outstanding is what has been requested behind those two (K fragments are
      // one request each, V fragments two).
      if (ch == 4) lds_wait2<2>(kf[4], kf[5]);        // behind them: kf6 kf7
      if (ch == 6) lds_wait2<4>(kf[6], kf[7]);        // vf0 vf1
      if (ch == 8) lds_wait2<4>(vf[0], vf[1]);        // vf2 vf3
      if (ch == 10) lds_wait2<4>(vf[2], vf[3]);       // vf4 vf5
      if (ch == 12) lds_wait2<4>(vf[4], vf[5]);       // vf6 vf7
      if (ch == 14) lds_wait2<2>(vf[6], vf[7]);       // kf0 kf1 of the next step
      auto mfma_of = [&](const int rt) {
        if (ch < 8) mfma_qk(ch, s_out[rt], rt);
        else mfma_pv(oacc[rt][(ch - 8) & 3], vf[ch - 8], p_in[rt][(ch - 8) >> 2]);
      };
      __builtin_amdgcn_sched_barrier(0);
      mfma_of(0);
      __builtin_amdgcn_sched_barrier(0);
      if (ch < 4) request_k(kaddr, 4 + ch);           // the LDS request of the chunk: the fragment needed four chunks on
      else if (ch < 12) request_v(vaddr, ch - 4);
      else request_k(knext, ch - 12);
      gap_work(2 * ch);
      __builtin_amdgcn_sched_barrier(0);
      mfma_of(1);
      __builtin_amdgcn_sched_barrier(0);
      gap_work(2 * ch + 1);
      if (par >= 0 && (ch & 3) == 1) issue(4 * par + (ch >> 2));      // this trip's share of the K/V stream
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int rt = 0; rt < NT; ++rt) {
      p_out[rt][0] = __builtin_bit_cast(bf16x8, uint4{packed[8 * rt + 0], packed[8 * rt + 1], packed[8 * rt + 2], packed[8 * rt + 3]});
      p_out[rt][1] = __builtin_bit_cast(bf16x8, uint4{packed[8 * rt + 4], packed[8 * rt + 5], packed[8 * rt + 6], packed[8 * rt + 7]});
    }
    // S^T of the next step stays allocated until its MFMAs have long retired, also when nobody reads it.
    // (Only then: where the next iteration reads it, the same statement makes the allocator copy all 32
    // registers behind every iteration.)
    if (par == -2) {
      asm volatile("" : "+v"(s_out[0]), "+v"(s_out[1]));
      return false;
    }
    return force || pending;      // wavefront-uniform
  };
  bool exact = true;
  if (active) {
    // S^T of step 0 against reference 0, then iteration 0 (exact prefix, no previous step)
#pragma unroll
    for (int i = 0; i < 8; ++i) request_k(k_slice(0), i);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      lds_wait1<0>(kf[i]);
      mfma_qk(i, sa[0], 0);
      mfma_qk(i, sa[1], 1);
    }
    mfma_settle(sa[0]);
    mfma_settle(sa[1]);
#pragma unroll
    for (int i = 0; i < 4; ++i) request_k(k_slice(1), i);
#pragma unroll
    for (int rt = 0; rt < NT; ++rt) {
      pb[rt][0] = pb[rt][1] = bf16x8{};
      asm volatile("" : "+v"(pb[rt][0]), "+v"(pb[rt][1]));
    }
    // iteration 0 has no previous step: its probabilities are zero and meet V of step 0, which is finite
    exact = iterate(true, -1, 0, k_slice(1), k_slice(0) + 16384, k_slice(2), sa, sb, pb, pa);
  }
  const int hshift = wave < 2 ? 5 : 4;
  auto hreq = [&](const int j) { return j + hshift; };
  auto end_trip = [&](const int j) {
    // K is consumed one trip ahead of V, so K(j + 5) and V(j + 4) replace what trip j has finished with;
    // they are issued during trip j + 1.  Only the eight loads issued during trip j may still be in flight.
    wait_vmcnt<8>();
    __builtin_amdgcn_s_barrier();
    setup_request(hreq(j));
  };
  end_trip(-1);
  int j = 0;
#pragma unroll 1
  for (; 2 * j + 2 < nsteps; ++j) {
    if (active) {
      // ring slots of half blocks j (V of this trip), j + 1 (K of this trip) and j + 2 (K fragments ahead)
      const unsigned s0 = lds_addr(smem) + (j & 3) * 32768, s1 = lds_addr(smem) + ((j + 1) & 3) * 32768,
                     s2 = lds_addr(smem) + ((j + 2) & 3) * 32768;
      exact = iterate(exact, 0, 2 * j + 1, s1, s0 + 16384, s1 + 8192, sb, sa, pa, pb);
      exact = iterate(exact, 1, 2 * j + 2, s1 + 8192, s0 + 16384 + 8192, s2, sa, sb, pb, pa);
      // no padding behind the last PV MFMAs here: the end of the trip (wait, barrier, next request) stands between
      // them and the next iteration, and the build-time check of the assembly would report a copy placed earlier
    } else {
#pragma unroll
      for (int idx = 0; idx < 8; ++idx) issue(idx);
    }
    end_trip(j);
  }
  if (2 * j + 1 < nsteps) {     // one more step: no refill (the last PV below still reads V of half block j)
    if (active) {
      iterate(exact, -2, 2 * j + 1, k_slice(2 * j + 2), k_slice(2 * j) + 16384, k_slice(2 * j + 3), sb, sa, pa, pb);
      settle_a(oacc[0][0], oacc[0][1], oacc[0][2], oacc[0][3]);
      settle_a(oacc[1][0], oacc[1][1], oacc[1][2], oacc[1][3]);
    }
  }
  if (active) {                 // PV of the last step
    lds_wait1<0>(kf[0]); lds_wait1<0>(kf[1]); lds_wait1<0>(kf[2]); lds_wait1<0>(kf[3]);
    const unsigned vaddr = k_slice(nsteps - 1) + 16384;
    const int last_keys = min(u.kv_end * kB, c.key_end) - jfirst - 32 * (nsteps - 1);     // keys of the last step: 1 .. 32
    if (last_keys < 32) zero_tail_rows(vaddr, last_keys, lane);
    bf16x8 p_last[NT][2];
#pragma unroll
    for (int rt = 0; rt < NT; ++rt) {
      p_last[rt][0] = (nsteps & 1) ? pa[rt][0] : pb[rt][0];
      p_last[rt][1] = (nsteps & 1) ? pa[rt][1] : pb[rt][1];
      asm volatile("" : "+v"(p_last[rt][0]), "+v"(p_last[rt][1]));     // selected here, not next to the MFMAs
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      request_v(vaddr, i);
      lds_wait1<0>(vf[i]);
      mfma_pv(oacc[0][i & 3], vf[i], p_last[0][i >> 2]);
      mfma_pv(oacc[1][i & 3], vf[i], p_last[1][i >> 2]);
    }
    ready_a(oacc[0][0], oacc[0][1], oacc[0][2], oacc[0][3]);
    ready_a(oacc[1][0], oacc[1][1], oacc[1][2], oacc[1][3]);
  }
  // The check of the optimistic pass.  All four wavefronts stream K/V together, so they repeat the unit together.
  bool bad = false;
  if (active) {
#pragma unroll
    for (int rt = 0; rt < NT; ++rt) {
      const float l_lane = (l_part[rt][0] + l_part[rt][1]) + (l_part[rt][2] + l_part[rt][3]);
      bad = bad || (r.valid[rt] && !(l_lane < kRowSumLimit));      // also true for NaN
    }
  }
  const bool wave_bad = __builtin_amdgcn_ballot_w64(bad) != 0;
  if (lane == 0) overflow_flags[wave] = wave_bad ? 1 : 0;
  __syncthreads();
  const int any_bad = overflow_flags[0] | overflow_flags[1] | overflow_flags[2] | overflow_flags[3];
  // The second pass is the caller's next turn of its loop over the units, not a loop in here: what a loop around
  // this function would keep alive across the main loop costs more registers than the wide units have to spare.
  if (__builtin_amdgcn_readfirstlane(any_bad) != 0 && !force) return true;
#pragma unroll
  for (int rt = 0; rt < NT; ++rt) {       // hand each 32-row tile to the single-tile epilogue
    Rows<1> r1;
    r1.lim[0] = r.lim[rt]; r1.tok[0] = r.tok[rt]; r1.valid[0] = r.valid[rt]; r1.mw0[0] = r.mw0[rt]; r1.mw1[0] = r.mw1[rt];
    UnitState st1;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) st1.oacc[0][dt] = oacc[rt][dt];
    // the epilogue expects the reference as a raw score and multiplies by c itself
    st1.m_ref[0] = m_ref[rt] == -INFINITY ? -INFINITY : (PRESCALE ? m_ref[rt] / cs : m_ref[rt]);
    st1.l_part[0] = (l_part[rt][0] + l_part[rt][1]) + (l_part[rt][2] + l_part[rt][3]);
    finish_unit(p, u, sq, c, r1, st1, row_base + 32 * rt, col, half);
  }
  return false;
}

// A unit with at most 32 rows (decode, short verify; bandwidth-bound): ONE wavefront processes the
// whole unit on its own, streaming 32-key slices through a private 16 KB ring (a K slot and a V slot,
// each refilled as soon as it has been consumed; a second slice in flight per wavefront was measured
// and gains nothing).  No barrier, no cross-wavefront merge: four such
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
      const int last_keys = min(u.kv_end * kB, c.key_end) - jfirst - 32 * t;      // keys of the last step: 1 .. 32
      if (last_keys < 32) zero_tail_rows(vaddr, last_keys, lane);
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
// wide units of its list together, then its four wavefronts draw the remaining (bandwidth-bound)
// units of the same list one by one from a shared cursor, each wavefront finishing whole units
// on its own.
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(1, 1))) void xy_attn_units_kernel(RunParams p) {
  __shared__ __attribute__((aligned(16))) unsigned char smem[4 * kTileBytes];
  __shared__ int cursor;
  __shared__ int overflow_flags[kThreads / 64];
  // consecutive workgroup ids land on different XCDs; give each XCD a contiguous range of workers
  int worker = blockIdx.x;
  if ((p.num_workers & 7) == 0) worker = (blockIdx.x & 7) * (p.num_workers >> 3) + (blockIdx.x >> 3);
  const int begin = as_const(p.worker_offsets)[worker], end = as_const(p.worker_offsets)[worker + 1];
  const LaneOffsets lo = make_lane_offsets(threadIdx.x & 63);
  const DmaOffsets dof = make_dma_offsets(threadIdx.x & 63, p.kv_ts);
  if (threadIdx.x == 0) cursor = begin;
  bool force = false;         // the unit at hand is run a second time, with exact references (see process_wide)
#pragma unroll 1
  for (int i = begin; i < end;) {
    const XyDevUnit u = load_const(p.units + i);
    if (u.q_count * u.head_count <= 32) {
      ++i;
      continue;
    }
    const XyDevSeq sq = load_const(p.seqs + u.seq);
    // Folding c into Q rounds q * c to bf16 once more; with the usual 1/sqrt(d) scale that is far inside the
    // tolerance, with a scale so large that scores reach tens of log2 units it is not, and c stays in fp32.
    bool again;
    if (p.kv_ts == kD) {
      if (p.c <= kPrescaleMaxC) again = process_wide<true, true>(p, u, sq, smem, overflow_flags, force, lo, dof);
      else again = process_wide<false, true>(p, u, sq, smem, overflow_flags, force, lo, dof);
    } else {
      if (p.c <= kPrescaleMaxC) again = process_wide<true, false>(p, u, sq, smem, overflow_flags, force, lo, dof);
      else again = process_wide<false, false>(p, u, sq, smem, overflow_flags, force, lo, dof);
    }
    force = again;              // wavefront- and workgroup-uniform
    if (!again) ++i;
  }
  __syncthreads();            // the tiles are free; the cursor is initialised
  // The narrow phase reads the kernel arguments afresh (through a pointer the compiler cannot see through)
  // instead of keeping the copies of the wide phase alive: what that phase had to spill to make room for
  // its own scalars would otherwise be reloaded lane by lane in every step of every narrow unit.
  const XY_CONST RunParams* args = (const XY_CONST RunParams*)__builtin_amdgcn_kernarg_segment_ptr();
  asm volatile("" : "+s"(args));
  const RunParams pn = load_const((const RunParams*)args);
#pragma unroll 1
  while (true) {
    int got = 0;
    if ((threadIdx.x & 63) == 0) got = atomicAdd(&cursor, 1);
    const int i = __builtin_amdgcn_readfirstlane(got);
    if (i >= end) break;
    const XyDevUnit u = load_const(pn.units + i);
    if (u.q_count * u.head_count > 32) continue;
    const XyDevSeq sq = load_const(pn.seqs + u.seq);
    process_solo(pn, u, sq, smem, lo, dof);
  }
  if (pn.counters) {
    // The shared list of narrow units (dynamic assignment): every wavefront of every workgroup draws the
    // next unit of the list, largest first, until it is empty.  The last workgroup to leave puts the
    // counters back to zero for the next launch (a plan runs one launch at a time, as its workspace does).
    // A wavefront's first unit is the one with its own slot number (wavefront x workers + worker), without
    // an atomic: a thousand wavefronts asking one counter at the same moment cost 15 us.
    const int shared_begin = as_const(pn.worker_offsets)[pn.num_workers];
    const int slots = pn.num_workers * (kThreads / 64);
    bool first = true;
#pragma unroll 1
    while (true) {
      int got = (threadIdx.x >> 6) * pn.num_workers + worker;   // wavefront-major: a short list still reaches every CU
      if (!first) {
        if (shared_begin + slots >= pn.num_units) break;       // one unit per wavefront was all there is
        got = 0;
        if ((threadIdx.x & 63) == 0) got = slots + atomicAdd(pn.counters, 1);
      }
      first = false;
      const int i = shared_begin + __builtin_amdgcn_readfirstlane(got);
      if (i >= pn.num_units) break;
      const XyDevUnit u = load_const(pn.units + i);
      const XyDevSeq sq = load_const(pn.seqs + u.seq);
      process_solo(pn, u, sq, smem, lo, dof);
    }
    __syncthreads();            // all four wavefronts are done with the cursor
    // No fence: every cursor draw above has returned its value, so it was performed at the
    // memory side before this count is; a device-wide fence here would write back and drop
    // this chiplet's L2 under the workgroups that are still streaming K/V through it.
    // The count of workgroups that have left is kept in two levels (eight groups of workgroups, each
    // on a cache line of its own, then one count of finished groups): 256 atomics on one address
    // would take several microseconds, which a short decode step cannot hide.
    if (threadIdx.x == 0) {
      const int groups = pn.num_workers < kDoneGroups ? pn.num_workers : kDoneGroups;
      const int g = worker % kDoneGroups;
      const int members = (pn.num_workers - g + kDoneGroups - 1) / kDoneGroups;
      int* done = pn.counters + kCounterStride * (1 + g);
      int* top = pn.counters + kCounterStride * (1 + kDoneGroups);
      if (atomicAdd(done, 1) == members - 1) {
        __hip_atomic_store(done, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (atomicAdd(top, 1) == groups - 1) {
          __hip_atomic_store(top, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          __hip_atomic_store(pn.counters, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
      }
    }
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

}  // namespace

// ---- the plan's tables on the GPU ---------------------------------------------------------------------
// One device arena and one pinned staging buffer per plan object, allocated when first needed, grown only when a
// rebuilt plan does not fit, freed with the plan.  A copy packs the tables into the staging buffer and enqueues
// ONE small copy kernel on the caller's stream; an event behind it says when the staging buffer
// may be written again.
void xy_plan_free_device(xy_attn_plan* plan) {
  if (!plan || plan->device < 0) return;
  int cur = 0;
  (void)hipGetDevice(&cur);
  (void)hipSetDevice(plan->device);
  if (plan->copied) {
    (void)hipEventSynchronize(static_cast<hipEvent_t>(plan->copied));
    (void)hipEventDestroy(static_cast<hipEvent_t>(plan->copied));
  }
  if (plan->d_arena) (void)hipFree(plan->d_arena);
  if (plan->h_stage) (void)hipHostFree(plan->h_stage);
  plan->d_arena = plan->h_stage = plan->h_stage_dev = plan->copied = nullptr;
  plan->d_units = plan->d_offsets = plan->d_seqs = plan->d_merges = plan->d_counters = nullptr;
  plan->arena_capacity = 0;
  plan->device = -1;
  plan->device_stale = true;
  (void)hipSetDevice(cur);
}

// 16 bytes per thread from the pinned staging buffer (read over the host link) to the arena
__global__ __launch_bounds__(256) void xy_plan_copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst,
                                                           unsigned chunks) {
  const unsigned i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < chunks) dst[i] = src[i];
}

static int plan_copy_to_device(xy_attn_plan* plan, hipStream_t stream) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return XY_ERR_HIP;
  if (plan->device >= 0 && plan->device != dev) return XY_ERR_ARG;      // the plan lives on another device
  auto round_up = [](size_t x) { return (x + 255) & ~(size_t)255; };
  const bool shared_list = plan->worker_offsets.back() < (int64_t)plan->units.size();
  const size_t off_units = 0;
  const size_t off_offsets = off_units + round_up(plan->units.size() * sizeof(XyDevUnit));
  const size_t off_seqs = off_offsets + round_up(plan->worker_offsets.size() * sizeof(int32_t));
  const size_t off_merges = off_seqs + round_up((size_t)plan->num_seqs * sizeof(XyDevSeq));
  const size_t off_counters = off_merges + round_up(plan->merges.size() * sizeof(xy_merge_item));
  const size_t need = off_counters + round_up(sizeof(int32_t) * kCounterStride * (kDoneGroups + 2));
  if (need > plan->arena_capacity) {
    xy_plan_free_device(plan);
    const size_t cap = std::max<size_t>(round_up(2 * need), (size_t)1 << 20);      // allocations are slow (milliseconds): grow rarely
    hipEvent_t ev = nullptr;
    if (hipMalloc(&plan->d_arena, cap) != hipSuccess || hipHostMalloc(&plan->h_stage, cap, hipHostMallocDefault) != hipSuccess ||
        hipEventCreateWithFlags(&ev, hipEventDisableTiming) != hipSuccess) {
      plan->device = dev;           // so that what was allocated is freed
      plan->copied = ev;
      xy_plan_free_device(plan);
      return XY_ERR_HIP;
    }
    plan->copied = ev;
    plan->arena_capacity = cap;
    plan->device = dev;
    if (hipHostGetDevicePointer(&plan->h_stage_dev, plan->h_stage, 0) != hipSuccess) {
      xy_plan_free_device(plan);
      return XY_ERR_HIP;
    }
  } else if (hipEventSynchronize(static_cast<hipEvent_t>(plan->copied)) != hipSuccess) {
    return XY_ERR_HIP;              // (the copy before this one has long finished in any sensible use)
  }
  unsigned char* h = static_cast<unsigned char*>(plan->h_stage);
  XyDevUnit* du = reinterpret_cast<XyDevUnit*>(h + off_units);
  for (size_t i = 0; i < plan->units.size(); ++i) {
    const xy_work_unit& u = plan->units[i];
    du[i] = XyDevUnit{u.seq, u.head_begin, u.head_count, u.q_begin, u.q_count,
                      u.kv_block_begin, u.kv_block_end, u.kind_flags, u.ws_offset};
  }
  memcpy(h + off_offsets, plan->worker_offsets.data(), plan->worker_offsets.size() * sizeof(int32_t));
  XyDevSeq* ds = reinterpret_cast<XyDevSeq*>(h + off_seqs);
  for (int32_t i = 0; i < plan->num_seqs; ++i) {
    const xy_seq_desc& s = plan->descs[i];
    ds[i] = XyDevSeq{s.query_len, s.context_len, plan->token_start[i], s.mask_kind, s.mask_word_offset};
  }
  if (!plan->merges.empty()) memcpy(h + off_merges, plan->merges.data(), plan->merges.size() * sizeof(xy_merge_item));
  memset(h + off_counters, 0, need - off_counters);       // cursor and finished-workgroup counts start at zero
  // The tables go over by a small kernel that reads the pinned buffer through its device mapping, not by the copy
  // engine: a copy-engine transfer in front of a kernel on the same stream costs about 0.15 ms of hand-over between
  // the two queues (measured: a serving step of 0.06 ms of kernels took 0.22 ms), a kernel-to-kernel order nothing.
  const unsigned chunks = (unsigned)(need / 16);
  hipLaunchKernelGGL(xy_plan_copy_kernel, dim3((chunks + 255) / 256), dim3(256), 0, stream,
                     static_cast<const uint4*>(plan->h_stage_dev), static_cast<uint4*>(plan->d_arena), chunks);
  if (hipGetLastError() != hipSuccess) return XY_ERR_HIP;
  if (hipEventRecord(static_cast<hipEvent_t>(plan->copied), stream) != hipSuccess) return XY_ERR_HIP;
  unsigned char* d = static_cast<unsigned char*>(plan->d_arena);
  plan->d_units = d + off_units;
  plan->d_offsets = d + off_offsets;
  plan->d_seqs = d + off_seqs;
  plan->d_merges = d + off_merges;
  plan->d_counters = shared_list ? d + off_counters : nullptr;
  plan->device_stale = false;
  return XY_OK;
}

extern "C" int xy_attn_plan_upload_async(xy_attn_plan* plan, void* hip_stream) {
  if (!plan) return XY_ERR_ARG;
  if (plan->device >= 0 && !plan->device_stale) return XY_OK;
  return plan_copy_to_device(plan, static_cast<hipStream_t>(hip_stream));
}

extern "C" int xy_attn_plan_upload(xy_attn_plan* plan) {
  if (!plan) return XY_ERR_ARG;
  if (plan->device >= 0 && !plan->device_stale) return XY_OK;
  if (int rc = plan_copy_to_device(plan, nullptr)) return rc;
  return hipStreamSynchronize(nullptr) == hipSuccess ? XY_OK : XY_ERR_HIP;
}

// Argument checks of a run (everything that can fail before device work is enqueued).
static int check_run_args(xy_attn_plan* plan, const void* q, int64_t q_ts, int64_t q_hs, const void* k_cache,
                          const void* v_cache, int64_t kv_bs, int64_t kv_hs, int64_t kv_ts,
                          const int32_t* block_table, const uint32_t* tree_masks, void* out, int64_t o_ts,
                          int64_t o_hs, void* workspace, size_t workspace_bytes, float softmax_scale,
                          hipStream_t stream) {
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
  if (int rc = xy_attn_plan_upload_async(plan, stream)) return rc;      // first use, or the plan was rebuilt since
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
                              out, o_ts, o_hs, workspace, workspace_bytes, softmax_scale,
                              static_cast<hipStream_t>(hip_stream)))
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
  p.num_units = (int32_t)plan->units.size();
  p.counters = static_cast<int32_t*>(plan->d_counters);
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
  if (int rc = xy_attn_plan_upload_async(plan, hip_stream)) return rc;
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

// ---- a run that allocates nothing -----------------------------------------------------------------------
// For callers that cannot allocate (a region under graph capture, a serving loop, a harness that forbids it):
// the partial results of K/V-split units go to a fixed array in device memory instead of a caller's workspace.
// Every GPU the library runs on holds its own copy of the array until the process ends.  In host code the
// array's name stands for the symbol, not for an address a kernel could use: the address on a device is asked
// for once, with that device current, and only that pointer is handed to the kernels.
constexpr size_t kScratchBytes = (size_t)XY_STATIC_WORKSPACE_BYTES;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_lock;
void* g_scratch_ptr[kMaxDevices] = {};      // per device, resolved on the first call there

int scratch_of_current_device(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return XY_ERR_HIP;
  std::lock_guard<std::mutex> hold(g_scratch_lock);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return XY_ERR_HIP;
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return XY_OK;
}
}  // namespace

extern "C" int xy_attn_run_static(xy_attn_plan* plan, const void* q, int64_t q_ts, int64_t q_hs, const void* k_cache,
                                  const void* v_cache, int64_t kv_bs, int64_t kv_hs, int64_t kv_ts,
                                  const int32_t* block_table, const uint32_t* tree_masks, void* out, int64_t o_ts,
                                  int64_t o_hs, float softmax_scale, void* hip_stream) {
  if (!plan) return XY_ERR_ARG;
  if ((size_t)plan->workspace_floats * sizeof(float) > kScratchBytes) return XY_ERR_WORKSPACE;
  if (plan->units.empty()) return XY_OK;
  if (plan->device < 0 || plan->device_stale) return XY_ERR_ARG;      // copying the plan to the GPU may allocate: xy_attn_plan_upload comes first
  void* ws = nullptr;
  if (int rc = scratch_of_current_device(&ws)) return rc;
  // The partial results need no initialisation: every split unit writes its whole partial before the merge reads it.
  return run_impl(XY_PHASE_UNITS | XY_PHASE_MERGE, plan, q, q_ts, q_hs, k_cache, v_cache, kv_bs, kv_hs, kv_ts,
                  block_table, tree_masks, out, o_ts, o_hs, ws, kScratchBytes, softmax_scale, hip_stream);
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
                              tree_masks, out, o_ts, o_hs, workspace, workspace_bytes, softmax_scale,
                              static_cast<hipStream_t>(hip_stream)))
    return rc;
  if (int rc = xy_attn_append_kv(plan, k_new, v_new, qkv_ts, qkv_hs, k_cache, v_cache, kv_bs, kv_hs, kv_ts,
                                 block_table, hip_stream))
    return rc;
  return run_impl(XY_PHASE_UNITS | XY_PHASE_MERGE, plan, qkv, qkv_ts, qkv_hs, k_cache, v_cache, kv_bs, kv_hs,
                  kv_ts, block_table, tree_masks, out, o_ts, o_hs, workspace, workspace_bytes, softmax_scale,
                  hip_stream);
}
