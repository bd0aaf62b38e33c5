// Prune + pack (Alg. 1 lines 6-7): per group keep the k elements of largest magnitude (ties: lowest index),
// store the kept values in ascending index order plus one bit per element.
//
// Three selection paths, chosen on the host from group_len:
//   1. wave-in-registers (group_len % 64 == 0, group_len <= 4096): one wavefront owns one group, holds it in
//      registers (lane l, slot j <-> element 64*j + l, so one wave ballot IS one 64-bit mask word), finds the
//      threshold from two LDS histogram levels and a few counting probes, then compacts with mbcnt prefix ranks.  The
//      activation is read from HBM exactly once and nothing but the packed result is written: select and pack are
//      fused.
//   2. wave-from-memory (other group_len <= 4096): same ownership, elements re-read from cache, bitwise search.
//   3. global (group_len > 4096, including the whole-tensor scope): MSB-first radix select with per-group digit
//      histograms in the workspace, then count / scan / pack kernels over 1024-element wave chunks.
// Paths 2 and 3 set mask bits with atomicOr on a zeroed mask because groups need not start on a word boundary.
// No floating-point arithmetic decides anything: keys are integer bit patterns, so results are bit-exact.
#include <vector>

#include "common.hpp"

namespace surgeon {

// ---------------------------------------------------------------------------------------------------------
// key handling.  "rot" form = magnitude bits shifted left by one with the sign bit moved to bit 0, so that
//   (rot >= 2*t)  <=>  (magnitude key >= t)   and the original bits are recoverable for the value store.
// ---------------------------------------------------------------------------------------------------------
template <typename BitsT>
struct Key;
template <>
struct Key<uint32_t> {
  static constexpr int kBits = 31;
  static constexpr uint32_t kMask = 0x7fffffffu;
  __device__ static __forceinline__ uint32_t rot(uint32_t b) { return (b << 1) | (b >> 31); }
  __device__ static __forceinline__ uint32_t unrot(uint32_t k) { return (k >> 1) | (k << 31); }
};
template <>
struct Key<uint16_t> {
  static constexpr int kBits = 15;
  static constexpr uint32_t kMask = 0x7fffu;
  // a 16-bit rotation: two copies of the value side by side, then one bit-field extract (two instructions)
  __device__ static __forceinline__ uint32_t rot(uint16_t b) {
    const uint32_t x = ((uint32_t)b << 16) | (uint32_t)b;
    return __builtin_amdgcn_ubfe(x, 15u, 16u);
  }
  // (the low 16 bits of (k << 15) | (k >> 1); one shift and one shift-or, tied down because the compiler otherwise
  // rewrites the pair as a 32-bit multiply, which runs at a quarter of the rate)
  __device__ static __forceinline__ uint16_t unrot(uint32_t k) {
    uint32_t r;
    asm("v_lshl_or_b32 %0, %1, 15, %2" : "=v"(r) : "v"(k), "v"(k >> 1));
    return (uint16_t)r;
  }
};

__device__ __forceinline__ uint64_t ballot64(bool p) { return __builtin_amdgcn_ballot_w64(p); }
// number of set bits of b below the calling lane, plus base
__device__ __forceinline__ uint32_t lane_rank(uint64_t b, uint32_t base) {
  return __builtin_amdgcn_mbcnt_hi((uint32_t)(b >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)b, base));
}
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v = max(v, (uint32_t)__shfl_xor((int)v, off, 64));
  return v;
}
// inclusive prefix sum inside each row of 16 lanes (DPP shifts, zero fill)
__device__ __forceinline__ uint32_t row_incl_scan_u32(uint32_t v) {
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x111, 0xf, 0xf, true);  // row_shr:1
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x112, 0xf, 0xf, true);  // row_shr:2
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x114, 0xf, 0xf, true);  // row_shr:4
  v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x118, 0xf, 0xf, true);  // row_shr:8
  return v;
}
// sum over the 64 lanes (wave-uniform result)
__device__ __forceinline__ uint32_t wave_sum_u32(uint32_t v) {
  v = row_incl_scan_u32(v);
  return (uint32_t)(__builtin_amdgcn_readlane((int)v, 15) + __builtin_amdgcn_readlane((int)v, 31) +
                    __builtin_amdgcn_readlane((int)v, 47) + __builtin_amdgcn_readlane((int)v, 63));
}
// inclusive prefix sum over the 64 lanes
__device__ __forceinline__ uint32_t wave_incl_scan_u32(uint32_t v, int lane) {
  v = row_incl_scan_u32(v);
  const uint32_t t0 = (uint32_t)__builtin_amdgcn_readlane((int)v, 15), t1 = (uint32_t)__builtin_amdgcn_readlane((int)v, 31),
                 t2 = (uint32_t)__builtin_amdgcn_readlane((int)v, 47);
  return v + (lane >= 16 ? t0 : 0u) + (lane >= 32 ? t1 : 0u) + (lane >= 48 ? t2 : 0u);
}
__device__ __forceinline__ uint64_t low_bits64(int q) { return q >= 64 ? ~0ull : (q <= 0 ? 0ull : ((1ull << q) - 1ull)); }

// Number of (slot, lane) pairs with rot key >= thr2.  Per-lane counters on the vector ALU, four independent
// compare -> add-with-carry chains per block so that no instruction waits for its predecessor; each compare
// result sits in its own SGPR pair and is consumed three instructions later (gfx940+ needs two wait states
// between a vector write of an SGPR and a vector read of it, which the compiler cannot add inside inline asm).
// Short groups (at most 16 slots) count with one ballot and a scalar popcount per slot instead: the per-lane counters
// end in a wave-wide sum (a DPP scan and four readlanes) whose cost no longer disappears behind a few slots.  For long
// groups the scalar route is no faster (measured: 4.5 against 5.0 TB/s on 4096-element groups): the scalar unit is
// shared by the four SIMDs of a compute unit and each pop-count waits for its compare.
template <int E>
__device__ __forceinline__ int count_ge(const uint32_t (&kr)[E], uint32_t thr2) {
  if constexpr (E % 4 == 0 && E > 16) {
    uint32_t c0 = 0, c1 = 0, c2 = 0, c3 = 0;
#pragma unroll
    for (int j = 0; j < E; j += 4) {
      uint64_t s0, s1, s2, s3;
      asm("v_cmp_ge_u32_e64 %[s0], %[k0], %[t]\n\t"
          "v_cmp_ge_u32_e64 %[s1], %[k1], %[t]\n\t"
          "v_cmp_ge_u32_e64 %[s2], %[k2], %[t]\n\t"
          "v_cmp_ge_u32_e64 %[s3], %[k3], %[t]\n\t"
          "v_addc_co_u32_e64 %[c0], %[s0], 0, %[c0], %[s0]\n\t"
          "v_addc_co_u32_e64 %[c1], %[s1], 0, %[c1], %[s1]\n\t"
          "v_addc_co_u32_e64 %[c2], %[s2], 0, %[c2], %[s2]\n\t"
          "v_addc_co_u32_e64 %[c3], %[s3], 0, %[c3], %[s3]"
          : [c0] "+v"(c0), [c1] "+v"(c1), [c2] "+v"(c2), [c3] "+v"(c3), [s0] "=&s"(s0), [s1] "=&s"(s1),
            [s2] "=&s"(s2), [s3] "=&s"(s3)
          : [k0] "v"(kr[j]), [k1] "v"(kr[j + 1]), [k2] "v"(kr[j + 2]), [k3] "v"(kr[j + 3]), [t] "v"(thr2));
    }
    return (int)wave_sum_u32((c0 + c1) + (c2 + c3));
  } else {
    int c = 0;
#pragma unroll
    for (int j = 0; j < E; ++j) c += __popcll(ballot64(kr[j] >= thr2));
    return c;
  }
}

// Lane J of (lo, hi) receives the ballot of slot J under the predicate (rot key >= thr), or > thr if STRICT.
template <int J, int E, bool STRICT>
struct CollectWords {
  __device__ static __forceinline__ void run(const uint32_t (&kr)[E], uint32_t thr, uint32_t& lo, uint32_t& hi) {
    if constexpr (J + 4 <= E) {
      uint64_t s0, s1, s2, s3;
      if constexpr (STRICT)
        asm volatile("v_cmp_gt_u32_e64 %0, %4, %8\n\tv_cmp_gt_u32_e64 %1, %5, %8\n\t"
                     "v_cmp_gt_u32_e64 %2, %6, %8\n\tv_cmp_gt_u32_e64 %3, %7, %8"
                     : "=&s"(s0), "=&s"(s1), "=&s"(s2), "=&s"(s3)
                     : "v"(kr[J]), "v"(kr[J + 1]), "v"(kr[J + 2]), "v"(kr[J + 3]), "v"(thr));
      else
        asm volatile("v_cmp_ge_u32_e64 %0, %4, %8\n\tv_cmp_ge_u32_e64 %1, %5, %8\n\t"
                     "v_cmp_ge_u32_e64 %2, %6, %8\n\tv_cmp_ge_u32_e64 %3, %7, %8"
                     : "=&s"(s0), "=&s"(s1), "=&s"(s2), "=&s"(s3)
                     : "v"(kr[J]), "v"(kr[J + 1]), "v"(kr[J + 2]), "v"(kr[J + 3]), "v"(thr));
      // volatile keeps these in order right behind the compares: each result is read >= 3 instructions after its write
      asm volatile("v_writelane_b32 %0, %2, %4\n\tv_writelane_b32 %1, %3, %4"
                   : "+v"(lo), "+v"(hi) : "s"((uint32_t)s0), "s"((uint32_t)(s0 >> 32)), "n"(J));
      asm volatile("v_writelane_b32 %0, %2, %4\n\tv_writelane_b32 %1, %3, %4"
                   : "+v"(lo), "+v"(hi) : "s"((uint32_t)s1), "s"((uint32_t)(s1 >> 32)), "n"(J + 1));
      asm volatile("v_writelane_b32 %0, %2, %4\n\tv_writelane_b32 %1, %3, %4"
                   : "+v"(lo), "+v"(hi) : "s"((uint32_t)s2), "s"((uint32_t)(s2 >> 32)), "n"(J + 2));
      asm volatile("v_writelane_b32 %0, %2, %4\n\tv_writelane_b32 %1, %3, %4"
                   : "+v"(lo), "+v"(hi) : "s"((uint32_t)s3), "s"((uint32_t)(s3 >> 32)), "n"(J + 3));
      CollectWords<J + 4, E, STRICT>::run(kr, thr, lo, hi);
    } else if constexpr (J < E) {
      const uint64_t b = ballot64(STRICT ? kr[J] > thr : kr[J] >= thr);
      asm volatile("s_nop 1\n\tv_writelane_b32 %0, %2, %4\n\tv_writelane_b32 %1, %3, %4"
                   : "+v"(lo), "+v"(hi) : "s"((uint32_t)b), "s"((uint32_t)(b >> 32)), "n"(J));
      CollectWords<J + 1, E, STRICT>::run(kr, thr, lo, hi);
    }
  }
};

// stores that drop out-of-range lanes in hardware: lanes that keep nothing pass offset 0xffffffff
__device__ __forceinline__ void store_or_drop(__amdgpu_buffer_rsrc_t rsrc, uint32_t v, uint32_t byte_off) {
  __builtin_amdgcn_raw_buffer_store_b32(v, rsrc, byte_off, 0, 0);
}
__device__ __forceinline__ void store_or_drop(__amdgpu_buffer_rsrc_t rsrc, uint16_t v, uint32_t byte_off) {
  __builtin_amdgcn_raw_buffer_store_b16(v, rsrc, byte_off, 0, 0);
}
constexpr int kBufferRsrcWord3 = 0x00020000;  // raw buffer, 32-bit data format (gfx9 family)

// Emits slot J: lane l stores its element at base(J) + (kept lanes below l) if bit l of keep word J is set.
// Every slot is independent of the others, so the stores stream at issue rate.
template <int J, int E, typename BitsT, bool WITH_IDX>
struct EmitSlots {
  __device__ static __forceinline__ void run(const uint32_t (&kr)[E], int lane, uint32_t w_lo, uint32_t w_hi, uint32_t base,
                                             __amdgpu_buffer_rsrc_t r_vals, __amdgpu_buffer_rsrc_t r_idx) {
    if constexpr (J < E) {
      const uint32_t b_lo = (uint32_t)__builtin_amdgcn_readlane((int)w_lo, J);
      const uint32_t b_hi = (uint32_t)__builtin_amdgcn_readlane((int)w_hi, J);
      const uint32_t base_j = (uint32_t)__builtin_amdgcn_readlane((int)base, J);
      const bool keep = __builtin_amdgcn_inverse_ballot_w64(((uint64_t)b_hi << 32) | b_lo);
      const uint32_t pos = __builtin_amdgcn_mbcnt_hi(b_hi, __builtin_amdgcn_mbcnt_lo(b_lo, base_j));
      store_or_drop(r_vals, Key<BitsT>::unrot(kr[J]), keep ? pos * (uint32_t)sizeof(BitsT) : 0xffffffffu);
      if constexpr (WITH_IDX) store_or_drop(r_idx, (uint32_t)(J * 64 + lane), keep ? pos * 4u : 0xffffffffu);
      EmitSlots<J + 1, E, BitsT, WITH_IDX>::run(kr, lane, w_lo, w_hi, base, r_vals, r_idx);
    }
  }
};

// Select and emit in one walk, for a threshold with exactly k keys at or above it: slot J's keep word comes from one
// compare, feeds the prefix ranks and the store directly, and lands in lane J of (w_lo, w_hi); `base` (kept elements of
// the earlier slots) is a scalar running count.  The two wait states that a vector read of a vector-written SGPR needs
// are spent inside the asm statement, wherever the compiler schedules it.
template <int J, int E, typename BitsT, bool WITH_IDX>
struct SelectEmitSlots {
  __device__ static __forceinline__ void run(const uint32_t (&kr)[E], int lane, uint32_t thr2, uint32_t base, uint32_t& w_lo,
                                             uint32_t& w_hi, __amdgpu_buffer_rsrc_t r_vals, __amdgpu_buffer_rsrc_t r_idx) {
    if constexpr (J < E) {
      const bool keep = kr[J] >= thr2;
      const uint64_t b = ballot64(keep);
      const uint32_t pos = lane_rank(b, base);
      store_or_drop(r_vals, Key<BitsT>::unrot(kr[J]), keep ? pos * (uint32_t)sizeof(BitsT) : 0xffffffffu);
      if constexpr (WITH_IDX) store_or_drop(r_idx, (uint32_t)(J * 64 + lane), keep ? pos * 4u : 0xffffffffu);
      asm volatile("s_nop 1\n\tv_writelane_b32 %0, %2, %4\n\tv_writelane_b32 %1, %3, %4"
                   : "+v"(w_lo), "+v"(w_hi) : "s"((uint32_t)b), "s"((uint32_t)(b >> 32)), "n"(J));
      SelectEmitSlots<J + 1, E, BitsT, WITH_IDX>::run(kr, lane, thr2, base + (uint32_t)__popcll(b), w_lo, w_hi, r_vals, r_idx);
    }
  }
};

// The same walk for a threshold key with ties: everything above the threshold magnitude is kept and, in index order,
// the first `need` elements equal to it.  Per slot two compares; whether the slot lies before the cut (keep its ties),
// behind it (drop them) or holds it (a scalar loop strips the surplus ties from the top, once per group) is decided on
// the scalar unit from the running count of ties, so no keep word makes the trip through a lane and back.
template <int J, int E, typename BitsT, bool WITH_IDX>
struct TieEmitSlots {
  __device__ static __forceinline__ void run(const uint32_t (&kr)[E], int lane, uint32_t thr2, uint32_t need, uint32_t eq_before,
                                             uint32_t base, uint32_t& w_lo, uint32_t& w_hi, __amdgpu_buffer_rsrc_t r_vals,
                                             __amdgpu_buffer_rsrc_t r_idx) {
    if constexpr (J < E) {
      const uint64_t b_ge = ballot64(kr[J] >= thr2);
      const uint64_t b_gt = ballot64(kr[J] > (thr2 | 1u));  // both signs of the threshold magnitude are ties
      const uint64_t eq = b_ge & ~b_gt;
      const uint32_t ce = (uint32_t)__popcll(eq);
      uint64_t b = b_ge;
      if (__builtin_expect(eq_before + ce > need, 0)) {
        uint64_t rest = eq;  // the ties of this slot that are not kept: all but its lowest need - eq_before
        for (uint32_t i = eq_before; i < need; ++i) rest &= rest - 1;
        b = b_ge & ~rest;
      }
      const bool keep = __builtin_amdgcn_inverse_ballot_w64(b);
      const uint32_t pos = lane_rank(b, base);
      store_or_drop(r_vals, Key<BitsT>::unrot(kr[J]), keep ? pos * (uint32_t)sizeof(BitsT) : 0xffffffffu);
      if constexpr (WITH_IDX) store_or_drop(r_idx, (uint32_t)(J * 64 + lane), keep ? pos * 4u : 0xffffffffu);
      asm volatile("s_nop 1\n\tv_writelane_b32 %0, %2, %4\n\tv_writelane_b32 %1, %3, %4"
                   : "+v"(w_lo), "+v"(w_hi) : "s"((uint32_t)b), "s"((uint32_t)(b >> 32)), "n"(J));
      TieEmitSlots<J + 1, E, BitsT, WITH_IDX>::run(kr, lane, thr2, need, eq_before + ce, base + (uint32_t)__popcll(b), w_lo,
                                                   w_hi, r_vals, r_idx);
    }
  }
};

// ---------------------------------------------------------------------------------------------------------
// Histogram seeding of the threshold search.  Counting probes cost two vector instructions per element
// each and about ten of them are needed from a cold start; a histogram over the top ten key bits costs about as much
// as one and a half probes (its additions run on the LDS, which this kernel does not otherwise use), and its bin
// counts, summed from the top, name the bin that holds the k-th largest key together with the exact counts at the
// bin's two ends.  A second histogram over the next ten bits of the keys inside that bin leaves a bracket of 2^11
// keys (fp32) or a single key (bf16) with exact counts at both ends, which the counting search then finishes -- often
// without a single probe, because the bracket's low end already has exactly k keys at or above it.  Measured on
// 4096-element fp32 groups: 38.6 -> 21.7 vector instructions per 64 elements, after which the kernel is no longer
// bound by vector issue (61 % busy) but by how much of its loads four wavefronts per SIMD can hide.  Short groups take
// it too: their cold-start search was a chain of scalar pop-counts and branches per probe (64-512-element bf16 groups:
// 0.88 -> 1.09 TB/s; 768-element groups +18 %).
// Zero keys are left out (count and position of the zeros follow from the total): a post-ReLU tensor would otherwise
// send half of its elements to one LDS address.
// ---------------------------------------------------------------------------------------------------------
constexpr int kHistBinBits = 10, kHistBins = 1 << kHistBinBits;

// One level: bins of (rot key >> shift) & bin_mask over the rot keys in [key_lo, key_lo + key_width) (modulo 2^32; one
// subtraction and one unsigned compare per key).  On return: bin = the bin that holds the want-th largest of those
// keys, above = how many of them lie in higher bins, inside = how many in the bin itself.  Returns false when fewer
// than `want` keys took part; above is then their number.  h: this wavefront's kHistBins words of LDS.
// BINS <= 64 (the second level of 16-bit keys has 32): one bin per lane, so a single word per lane is cleared and read
// back and one wavefront scan finds the bin.
template <int E, bool ALL_NONZERO, int BINS = kHistBins>  // ALL_NONZERO: key_lo = 2, the range runs to the top (level 1)
__device__ __forceinline__ bool hist_level(const uint32_t (&kr)[E], uint32_t* h, int lane, int shift, uint32_t bin_mask,
                                           uint32_t key_lo, uint32_t key_width, uint32_t want, uint32_t* bin,
                                           uint32_t* above, uint32_t* inside) {
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  u32x4* h4 = reinterpret_cast<u32x4*>(h);
  static_assert(BINS == kHistBins || BINS <= 64, "either the full table or one bin per lane");
  if constexpr (BINS <= 64) {
    h[lane] = 0u;
  } else {
#pragma unroll
    for (int i = 0; i < kHistBins / 256; ++i) h4[lane + 64 * i] = u32x4{0u, 0u, 0u, 0u};
  }
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  // The additions: per key one shift, one and-or (bin -> LDS byte address; the wavefront's region is 4 KB aligned), a
  // compare that narrows exec to the keys that take part, and the LDS add -- the last two inside one asm statement
  // that puts exec back, so the compiler sees no change of it.  (From C++ the same loop compiled to six vector
  // instructions per key and cost as much as the probes it replaces.)  LDS instructions of a wavefront execute in
  // order, so the reads below see the additions.
  uint32_t base;  // in a vector register, so that mask (scalar) and base fit one and-or instruction
  asm("v_mov_b32 %0, %1" : "=v"(base) : "s"((uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint32_t*)h));
  const uint32_t one = 1u, byte_mask = bin_mask << 2;
#pragma unroll
  for (int j = 0; j < E; ++j) {
    const uint32_t addr = ((shift >= 2 ? kr[j] >> (shift - 2) : kr[j] << (2 - shift)) & byte_mask) | base;
    uint64_t saved;
    if constexpr (ALL_NONZERO)
      asm volatile("s_mov_b64 %0, exec\n\tv_cmpx_le_u32_e32 2, %1\n\tds_add_u32 %2, %3\n\ts_mov_b64 exec, %0"
                   : "=&s"(saved) : "v"(kr[j]), "v"(addr), "v"(one) : "vcc", "memory");
    else
      asm volatile("s_mov_b64 %0, exec\n\tv_cmpx_gt_u32_e32 %1, %2\n\tds_add_u32 %3, %4\n\ts_mov_b64 exec, %0"
                   : "=&s"(saved) : "s"(key_width), "v"(kr[j] - key_lo), "v"(addr), "v"(one) : "vcc", "memory");
  }
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  if constexpr (BINS <= 64) {
    // lane l holds bin 63 - l (bins from BINS up were cleared and never added to)
    const uint32_t c = h[63 - lane];
    const uint32_t incl = wave_incl_scan_u32(c, lane);
    const uint64_t has = ballot64(incl >= want);
    if (has == 0) {
      *above = (uint32_t)__builtin_amdgcn_readlane((int)incl, 63);
      return false;
    }
    const int L = __builtin_ctzll(has);
    *bin = (uint32_t)(63 - L);
    *inside = (uint32_t)__builtin_amdgcn_readlane((int)c, L);
    *above = (uint32_t)__builtin_amdgcn_readlane((int)incl, L) - *inside;
    return true;
  }
  // lane l sums the 16 bins of chunk 63 - l, so that a prefix sum over the lanes runs from the highest keys down
  uint32_t s = 0;
#pragma unroll
  for (int i = 0; i < kHistBins / 256; ++i) {
    const u32x4 q = h4[(63 - lane) * (kHistBins / 256) + i];
    s += (q[0] + q[1]) + (q[2] + q[3]);
  }
  const uint32_t incl = wave_incl_scan_u32(s, lane);
  const uint64_t has = ballot64(incl >= want);
  if (has == 0) {
    *above = (uint32_t)__builtin_amdgcn_readlane((int)incl, 63);
    return false;
  }
  const int L = __builtin_ctzll(has);  // first lane, from the top, whose chunk reaches the want-th key
  const uint32_t before = (uint32_t)__builtin_amdgcn_readlane((int)(incl - s), L);
  // the chunk's 16 bins, highest first, on lanes 0..15 (every row of 16 lanes does the same)
  const int chunk = 63 - L;
  const uint32_t c = h[chunk * 16 + 15 - (lane & 15)];
  const uint32_t run = row_incl_scan_u32(c) + before;
  const uint64_t hit = ballot64(run >= want) & 0xffffull;
  const int i = __builtin_ctzll(hit);  // non-empty: the chunk's total reaches want
  *bin = (uint32_t)(chunk * 16 + 15 - i);
  *inside = (uint32_t)__builtin_amdgcn_readlane((int)c, i);
  *above = (uint32_t)__builtin_amdgcn_readlane((int)run, i) - *inside;
  return true;
}

// ---------------------------------------------------------------------------------------------------------
// path 1: one wavefront per group, group in registers
// ---------------------------------------------------------------------------------------------------------
// group `grp` of one tensor, by the calling wavefront
template <int E, typename BitsT, bool WITH_IDX>
__device__ __forceinline__ void select_pack_group(const BitsT* __restrict__ A, BitsT* __restrict__ vals,
                                                  uint64_t* __restrict__ mask, uint32_t* __restrict__ idx, int64_t grp,
                                                  int64_t n_groups, int g, int len_last, int k_full, int k_last) {
  const int lane = threadIdx.x & 63;
  const bool is_last = grp == n_groups - 1;
  const int len = is_last ? len_last : g;
  const int k = is_last ? k_last : k_full;
  const int64_t gstart = grp * (int64_t)g;
  const BitsT* __restrict__ src = A + gstart;

  // lane l, slot j <-> element 64*j + l.  All loads are issued before the first use.  A short group re-reads
  // its last element for the missing slots, which then become magnitude 0 at the highest indices.
  uint32_t kr[E];
  if (len == E * 64) {
#pragma unroll
    for (int j = 0; j < E; ++j) kr[j] = (uint32_t)__builtin_nontemporal_load(&src[j * 64 + lane]);
#pragma unroll
    for (int j = 0; j < E; ++j) kr[j] = Key<BitsT>::rot((BitsT)kr[j]);
  } else {
#pragma unroll
    for (int j = 0; j < E; ++j) kr[j] = (uint32_t)__builtin_nontemporal_load(&src[min(j * 64 + lane, len - 1)]);
#pragma unroll
    for (int j = 0; j < E; ++j) kr[j] = (j * 64 + lane < len) ? Key<BitsT>::rot((BitsT)kr[j]) : 0u;
  }

  // ---- the keep words: lane j of (w_lo, w_hi) = mask word j of this group
  uint32_t w_lo = 0, w_hi = 0;
  if (k >= len) {
    const uint64_t w = lane < E ? low_bits64(len - 64 * lane) : 0ull;
    w_lo = (uint32_t)w;
    w_hi = (uint32_t)(w >> 32);
  } else {
    // invariant: count(key >= lo) >= k and count(key >= hi) < k, so the k-th largest key is in [lo, hi).
    // f_lo = count(lo) - k >= 0 and f_hi = count(hi) - k < 0 drive a regula-falsi search on the integer key;
    // when one end moves twice in a row the other end's weight is halved (Illinois rule), so the bracket
    // shrinks super-linearly on smooth distributions and at least geometrically on plateaus of ties.
    uint32_t lo = 0, hi = 1;
    float f_lo = 0.0f, f_hi = 0.0f;
    int c_hi = 0;
    bool found = false;
    uint32_t thr2 = 0;
    {
      // two histogram levels put the bracket around the k-th largest key with exact counts at both ends
      __shared__ __attribute__((aligned(16))) uint32_t hist_lds[4][kHistBins];
      uint32_t* h = hist_lds[__builtin_amdgcn_readfirstlane(threadIdx.x >> 6)];
      constexpr int S1 = Key<BitsT>::kBits + 1 - kHistBinBits;              // rot keys have kBits + 1 bits
      constexpr int S2 = S1 - kHistBinBits > 1 ? S1 - kHistBinBits : 1;     // bit 0 is the sign
      uint32_t b1 = 0, above1 = 0, in1 = 0;
      // level 1: every key of non-zero magnitude (rot key >= 2)
      if (!hist_level<E, true>(kr, h, lane, S1, (uint32_t)(kHistBins - 1), 2u, 0u - 2u, (uint32_t)k, &b1, &above1, &in1)) {
        // fewer than k non-zero keys: the threshold is the tie at zero (lo = 0, hi = 1), and count(key >= 1) is the
        // histogram's total
        c_hi = (int)above1;
      } else {
        // level 2: the non-zero keys of bin b1 (at least k - above1 of them), by their next S1 - S2 bits
        uint32_t b2 = 0, above2 = 0, in2 = 0;
        const uint32_t bin_lo = max(b1 << S1, 2u);
        constexpr int kBins2 = (1 << (S1 - S2)) <= 64 ? (1 << (S1 - S2)) : kHistBins;
        hist_level<E, false, kBins2>(kr, h, lane, S2, (1u << (S1 - S2)) - 1u, bin_lo, ((b1 + 1u) << S1) - bin_lo,
                             (uint32_t)k - above1, &b2, &above2, &in2);
        const uint32_t lo_rot = (b1 << S1) | (b2 << S2);
        lo = max(lo_rot >> 1, 1u);  // the histogram holds no zero keys: its lowest bin starts at magnitude 1
        hi = (lo_rot >> 1) + (1u << (S2 - 1));
        c_hi = (int)(above1 + above2);
        const int c_lo = c_hi + (int)in2;
        f_lo = (float)(c_lo - k);
        f_hi = (float)(c_hi - k);
        if (c_lo == k) {
          found = true;
          thr2 = lo << 1;
        }
      }
    }
    int last_side = 0;  // +1: lo moved last, -1: hi moved last
    while (!found && hi - lo > 1) {
      const uint32_t span = hi - lo;
      uint32_t d = (uint32_t)(f_lo * __builtin_amdgcn_rcpf(f_lo - f_hi) * (float)span);
      d = min(max(d, 1u), span - 1u);
      const uint32_t mid = lo + d;
      const int c = count_ge<E>(kr, mid << 1);
      if (c == k) {
        found = true;
        thr2 = mid << 1;
      } else if (c > k) {
        lo = mid;
        f_lo = (float)(c - k);
        if (last_side > 0) f_hi *= 0.5f;
        last_side = 1;
      } else {
        hi = mid;
        c_hi = c;
        f_hi = (float)(c - k);
        if (last_side < 0) f_lo *= 0.5f;
        last_side = -1;
      }
    }
    if (found) {
      // exactly k keys are >= thr2: no tie to resolve, so each slot's keep word goes from its compare straight into the
      // pack (prefix ranks inside the slot, a scalar running count for the slot's base) and into lane j of the mask words
      const __amdgpu_buffer_rsrc_t r_vals = __builtin_amdgcn_make_buffer_rsrc(
          vals + grp * (int64_t)k_full, 0, k * (int)sizeof(BitsT), kBufferRsrcWord3);
      const __amdgpu_buffer_rsrc_t r_idx = __builtin_amdgcn_make_buffer_rsrc(
          WITH_IDX ? idx + grp * (int64_t)k_full : (uint32_t*)nullptr, 0, WITH_IDX ? k * 4 : 0, kBufferRsrcWord3);
      SelectEmitSlots<0, E, BitsT, WITH_IDX>::run(kr, lane, thr2, 0u, w_lo, w_hi, r_vals, r_idx);
      const int n_words = (len + 63) >> 6;
      if (lane < n_words) mask[(gstart >> 6) + lane] = ((uint64_t)w_hi << 32) | w_lo;
      return;
    } else {
      // hi == lo + 1: more than k keys are >= lo, fewer than k are > lo.  Keep everything above the threshold key
      // and the first `need` elements equal to it in index order.
      thr2 = lo << 1;
      const uint32_t need = (uint32_t)(k - c_hi);
      if constexpr (sizeof(BitsT) == 2) {
        // 16-bit keys: a 4096-element group has several elements per key value around its threshold, so this is the
        // usual way out and gets the one-walk form (ResNet-50 / ViT / segmentation workloads +1-4 %)
        const __amdgpu_buffer_rsrc_t r_vals = __builtin_amdgcn_make_buffer_rsrc(
            vals + grp * (int64_t)k_full, 0, k * (int)sizeof(BitsT), kBufferRsrcWord3);
        const __amdgpu_buffer_rsrc_t r_idx = __builtin_amdgcn_make_buffer_rsrc(
            WITH_IDX ? idx + grp * (int64_t)k_full : (uint32_t*)nullptr, 0, WITH_IDX ? k * 4 : 0, kBufferRsrcWord3);
        TieEmitSlots<0, E, BitsT, WITH_IDX>::run(kr, lane, thr2, need, 0u, 0u, w_lo, w_hi, r_vals, r_idx);
        const int n_words = (len + 63) >> 6;
        if (lane < n_words) mask[(gstart >> 6) + lane] = ((uint64_t)w_hi << 32) | w_lo;
        return;
      } else {
        // 32-bit keys: ties are the exception (a plateau of zeros behind a ReLU, a clipped maximum); the keep words are
        // collected on the lanes, the cut is found there, and the generic pack below emits them (the one-walk form
        // here made the kernel a third longer and the headline workload 1 % slower)
        uint32_t gt_lo = 0, gt_hi = 0;
        CollectWords<0, E, false>::run(kr, thr2, w_lo, w_hi);      // >= threshold
        CollectWords<0, E, true>::run(kr, thr2 | 1u, gt_lo, gt_hi);  // >  threshold (both signs share thr2 | 1)
        const uint64_t eq = (((uint64_t)w_hi << 32) | w_lo) & ~(((uint64_t)gt_hi << 32) | gt_lo);
        const uint32_t ce = (uint32_t)__popcll(eq);
        const uint32_t e_incl = wave_incl_scan_u32(ce, lane), e_base = e_incl - ce;  // tied elements in earlier slots
        if (e_incl > need) {  // not all of this slot's tied elements are kept
          uint64_t keep_eq = 0;
          if (e_base < need) {  // the cut falls inside this slot (at most one lane): its lowest need - e_base tied bits
            const uint32_t want = need - e_base;
            int p = 0;
#pragma unroll
            for (int step = 32; step >= 1; step >>= 1)
              if ((uint32_t)__popcll(eq & low_bits64(p + step)) < want) p += step;
            keep_eq = eq & low_bits64(p + 1);
          }
          w_lo = gt_lo | (uint32_t)keep_eq;
          w_hi = gt_hi | (uint32_t)(keep_eq >> 32);
        }
      }
    }
  }

  // ---- pack: slot bases from a prefix sum over the lanes holding the words, then independent slot stores
  const uint32_t kept = (uint32_t)__builtin_popcount(w_lo) + (uint32_t)__builtin_popcount(w_hi);
  const uint32_t base = wave_incl_scan_u32(kept, lane) - kept;
  const __amdgpu_buffer_rsrc_t r_vals = __builtin_amdgcn_make_buffer_rsrc(
      vals + grp * (int64_t)k_full, 0, k * (int)sizeof(BitsT), kBufferRsrcWord3);
  const __amdgpu_buffer_rsrc_t r_idx = __builtin_amdgcn_make_buffer_rsrc(
      WITH_IDX ? idx + grp * (int64_t)k_full : (uint32_t*)nullptr, 0, WITH_IDX ? k * 4 : 0, kBufferRsrcWord3);
  EmitSlots<0, E, BitsT, WITH_IDX>::run(kr, lane, w_lo, w_hi, base, r_vals, r_idx);
  const int n_words = (len + 63) >> 6;
  if (lane < n_words) mask[(gstart >> 6) + lane] = ((uint64_t)w_hi << 32) | w_lo;
}

// Wavefronts per SIMD the register allocation aims for.  Since the histogram seeding the kernel is no longer bound by
// vector issue and a fifth wavefront hides more of the loads: measured +7 % on the bf16 workloads; the fp32 headline
// workload is 1 % faster with four (128 registers).
template <typename BitsT>
constexpr int kSelectWaves = sizeof(BitsT) == 2 ? 5 : 4;

template <int E, typename BitsT, bool WITH_IDX>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(kSelectWaves<BitsT>))) void select_pack_wave_reg_kernel(const BitsT* __restrict__ A,
                                                                   BitsT* __restrict__ vals,
                                                                   uint64_t* __restrict__ mask,
                                                                   uint32_t* __restrict__ idx, int64_t n_groups,
                                                                   int g, int len_last, int k_full, int k_last) {
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int64_t grp = (int64_t)blockIdx.x * 4 + wave;
  if (grp >= n_groups) return;
  select_pack_group<E, BitsT, WITH_IDX>(A, vals, mask, idx, grp, n_groups, g, len_last, k_full, k_last);
}

// ---- many tensors in one launch (surgeon_prune_pack_batched): the tensors of a network are small next to the chip
// (a layer of 8 M elements is two rounds of wavefronts), so per-tensor launches pay a launch gap and a ragged tail each.
// The descriptors of up to kPackBatch tensors travel as kernel arguments; workgroup -> tensor by its first workgroup.
constexpr int kPackBatch = 48;
struct PackBatch {
  const void* A[kPackBatch];
  void* vals[kPackBatch];
  uint64_t* mask[kPackBatch];
  int64_t n_groups[kPackBatch];
  int first_block[kPackBatch + 1];  // workgroups [first_block[i], first_block[i+1]) belong to tensor i
  int g[kPackBatch], len_last[kPackBatch], k_full[kPackBatch], k_last[kPackBatch];
};

template <int E, typename BitsT>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(kSelectWaves<BitsT>))) void select_pack_wave_reg_batched_kernel(PackBatch bt) {
  // the tensor of this workgroup = the last boundary at or below its index, by a branch-free binary search whose six
  // steps are scalar loads from the argument block (47 independent compares compile to a compare, a select and a lane
  // read each: a fifth of the vector instructions of a 768-element group); entries past the last tensor hold the
  // total, which no index reaches
  int t = 0;
#pragma unroll
  for (int step = 32; step >= 1; step >>= 1) {
    const int c = min(t + step, kPackBatch);
    t = (int)blockIdx.x >= bt.first_block[c] ? c : t;
  }
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int64_t grp = (int64_t)((int)blockIdx.x - bt.first_block[t]) * 4 + wave;
  if (grp >= bt.n_groups[t]) return;
  select_pack_group<E, BitsT, false>((const BitsT*)bt.A[t], (BitsT*)bt.vals[t], bt.mask[t], (uint32_t*)nullptr, grp,
                                     bt.n_groups[t], bt.g[t], bt.len_last[t], bt.k_full[t], bt.k_last[t]);
}

// ---------------------------------------------------------------------------------------------------------
// shared by paths 2 and 3
// ---------------------------------------------------------------------------------------------------------
__global__ void fill_zero_u64_kernel(uint64_t* __restrict__ p, int64_t n) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) p[i] = 0;
}

// OR the ballot of 64 consecutive elements starting at flat index e_first into the (zeroed) mask
__device__ __forceinline__ void or_into_mask(uint64_t* __restrict__ mask, int64_t e_first, uint64_t b, int lane) {
  if (lane == 0 && b) {
    const int64_t w = e_first >> 6;
    const int sh = (int)(e_first & 63);
    atomicOr((unsigned long long*)&mask[w], (unsigned long long)(b << sh));
    if (sh) {
      const uint64_t hi_part = b >> (64 - sh);
      if (hi_part) atomicOr((unsigned long long*)&mask[w + 1], (unsigned long long)hi_part);
    }
  }
}

// ---------------------------------------------------------------------------------------------------------
// path 2: one wavefront per group, elements re-read from memory (any group_len; used for group_len <= 4096)
// ---------------------------------------------------------------------------------------------------------
template <typename BitsT, bool WITH_IDX>
__global__ __launch_bounds__(256) void select_pack_wave_mem_kernel(const BitsT* __restrict__ A,
                                                                   BitsT* __restrict__ vals,
                                                                   uint64_t* __restrict__ mask,
                                                                   uint32_t* __restrict__ idx, int64_t n_groups,
                                                                   int g, int len_last, int k_full, int k_last) {
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int64_t grp = (int64_t)blockIdx.x * 4 + wave;
  if (grp >= n_groups) return;
  const bool is_last = grp == n_groups - 1;
  const int len = is_last ? len_last : g;
  const int k = is_last ? k_last : k_full;
  const int64_t gstart = grp * (int64_t)g;
  const BitsT* __restrict__ src = A + gstart;

  // largest t with count(key >= t) >= k, one bit at a time from the top: the k-th largest key
  uint32_t t_key = 0;
  for (int bit = Key<BitsT>::kBits - 1; bit >= 0; --bit) {
    const uint32_t cand = t_key | (1u << bit);
    int c = 0;
    for (int base = 0; base < len; base += 64) {
      const int pos = base + lane;
      const bool p = pos < len && ((uint32_t)src[pos] & Key<BitsT>::kMask) >= cand;
      c += __popcll(ballot64(p));
    }
    if (c >= k) t_key = cand;
  }
  int c_gt = 0;
  for (int base = 0; base < len; base += 64) {
    const int pos = base + lane;
    c_gt += __popcll(ballot64(pos < len && ((uint32_t)src[pos] & Key<BitsT>::kMask) > t_key));
  }
  const uint32_t need = (uint32_t)(k - c_gt);

  BitsT* __restrict__ out_vals = vals + grp * (int64_t)k_full;
  uint32_t* __restrict__ out_idx = WITH_IDX ? idx + grp * (int64_t)k_full : nullptr;
  uint32_t run = 0, eq_run = 0;
  for (int base = 0; base < len; base += 64) {
    const int pos = base + lane;
    const bool valid = pos < len;
    const BitsT bits = valid ? src[pos] : (BitsT)0;
    const uint32_t key = (uint32_t)bits & Key<BitsT>::kMask;
    const bool gt = valid && key > t_key;
    const bool eq = valid && key == t_key;
    const uint64_t beq = ballot64(eq);
    const bool keep = gt || (eq && lane_rank(beq, eq_run) < need);
    const uint64_t b = ballot64(keep);
    if (keep) {
      const uint32_t o = lane_rank(b, run);
      out_vals[o] = bits;
      if (WITH_IDX) out_idx[o] = (uint32_t)pos;
    }
    or_into_mask(mask, gstart + base, b, lane);
    run += (uint32_t)__popcll(b);
    eq_run += (uint32_t)__popcll(beq);
  }
}

// ---------------------------------------------------------------------------------------------------------
// path 3: groups larger than one wavefront can hold -- radix select over HBM with workspace state
// ---------------------------------------------------------------------------------------------------------
struct GroupState {
  uint32_t prefix;  // digits of the threshold key fixed so far
  uint32_t k_rem;   // rank still to resolve among elements matching the prefix
  uint32_t t_key;   // final threshold key
  uint32_t need;    // elements equal to t_key that are kept
};

__global__ void gsel_init_kernel(GroupState* __restrict__ st, uint32_t* __restrict__ hist, int64_t n_groups,
                                 uint32_t k_full, uint32_t k_last, int replicas) {
  const int64_t tid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t i = tid; i < n_groups * replicas * kGlobalHistBins; i += stride) hist[i] = 0;
  for (int64_t i = tid; i < n_groups; i += stride) {
    GroupState s;
    s.prefix = 0;
    s.k_rem = (i == n_groups - 1) ? k_last : k_full;
    s.t_key = 0;
    s.need = 0;
    st[i] = s;
  }
}

// One digit pass: histogram of the digit at `shift` over the elements whose higher bits match the prefix.
// A workgroup histograms kGlobalHistChunk elements in LDS and adds its non-empty bins to the group's histogram.
// Lanes whose digit is 0 (in the first pass: every exact zero of a post-ReLU tensor) are counted with one ballot
// per load instead of one LDS atomic each, which would all hit the same address.
template <typename BitsT>
__global__ __launch_bounds__(256) void gsel_hist_kernel(const BitsT* __restrict__ A, int64_t n, int64_t g,
                                                        int64_t blocks_per_group, int shift, int nbits,
                                                        const GroupState* __restrict__ st,
                                                        uint32_t* __restrict__ hist, int replicas) {
  __shared__ uint32_t lh[kGlobalHistBins];
  const int64_t grp = blockIdx.x / blocks_per_group;
  const int64_t blk = blockIdx.x % blocks_per_group;
  for (int b = threadIdx.x; b < kGlobalHistBins; b += 256) lh[b] = 0;
  __syncthreads();
  const int64_t gstart = grp * g;
  const int64_t gend = min(gstart + g, n);
  const int64_t e0 = gstart + blk * kGlobalHistChunk;
  const int hshift = shift + nbits;
  const uint32_t want = hshift >= 32 ? 0u : (st[grp].prefix >> hshift);
  const uint32_t dmask = (1u << nbits) - 1u;
  const int lane = threadIdx.x & 63;
  uint32_t zeros = 0;  // elements of this wavefront with digit 0 (wave-uniform)
  constexpr int kBatch = 8;
  for (int t0 = 0; t0 < kGlobalHistChunk; t0 += 256 * kBatch) {
    uint32_t key[kBatch];
    bool ok[kBatch];
#pragma unroll
    for (int q = 0; q < kBatch; ++q) {
      const int64_t e = e0 + t0 + q * 256 + threadIdx.x;
      ok[q] = e < gend;
      key[q] = (uint32_t)A[ok[q] ? e : gend - 1] & Key<BitsT>::kMask;
    }
#pragma unroll
    for (int q = 0; q < kBatch; ++q) {
      const bool match = ok[q] && (hshift >= 32 || (key[q] >> hshift) == want);
      const uint32_t digit = (key[q] >> shift) & dmask;
      zeros += (uint32_t)__popcll(ballot64(match && digit == 0u));
      if (match && digit != 0u) atomicAdd(&lh[digit], 1u);
    }
  }
  if (lane == 0 && zeros) atomicAdd(&lh[0], zeros);
  __syncthreads();
  uint32_t* __restrict__ h = hist + (grp * replicas + blk % replicas) * (int64_t)kGlobalHistBins;
  for (int b = threadIdx.x; b < kGlobalHistBins; b += 256) {
    const uint32_t c = lh[b];
    if (c) atomicAdd(&h[b], c);
  }
}

// exclusive prefix sum over the threads of a workgroup of up to 1024 threads (lds17: 17 words); *total = the sum
__device__ __forceinline__ uint32_t block_excl_scan(uint32_t v, uint32_t* lds17, uint32_t* total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, n_waves = (blockDim.x + 63) >> 6;
  const uint32_t incl = wave_incl_scan_u32(v, lane);
  __syncthreads();  // lds17 may still be read from the previous call
  if (lane == 63) lds17[wave] = incl;
  __syncthreads();
  if (threadIdx.x == 0) {
    uint32_t acc = 0;
    for (int w = 0; w < n_waves; ++w) {
      const uint32_t x = lds17[w];
      lds17[w] = acc;
      acc += x;
    }
    lds17[16] = acc;
  }
  __syncthreads();
  *total = lds17[16];
  return lds17[wave] + incl - v;
}

// Picks the digit holding the k_rem-th largest matching element and clears the histogram for the next pass.
// The group's histogram exists in `replicas` copies (workgroups of the histogram pass spread their atomics over
// them); they are summed here.
__global__ __launch_bounds__(256) void gsel_resolve_kernel(GroupState* __restrict__ st, uint32_t* __restrict__ hist,
                                                           int replicas, int shift, int last) {
  constexpr int kPer = kGlobalHistBins / 256;  // consecutive bins per thread
  __shared__ uint32_t lds17[17];
  const int64_t grp = blockIdx.x;
  const int tid = threadIdx.x;
  uint32_t* __restrict__ h = hist + grp * replicas * (int64_t)kGlobalHistBins;
  uint32_t c[kPer];
  uint32_t sum = 0;
#pragma unroll
  for (int q = 0; q < kPer; ++q) c[q] = 0;
  for (int rep = 0; rep < replicas; ++rep) {
#pragma unroll
    for (int q = 0; q < kPer; ++q) {
      c[q] += h[rep * kGlobalHistBins + tid * kPer + q];
      h[rep * kGlobalHistBins + tid * kPer + q] = 0;
    }
  }
#pragma unroll
  for (int q = 0; q < kPer; ++q) sum += c[q];
  const GroupState s = st[grp];
  uint32_t total;
  const uint32_t below = block_excl_scan(sum, lds17, &total);
  uint32_t above = total - below - sum;  // matching elements in the bins above this thread's
#pragma unroll
  for (int q = kPer - 1; q >= 0; --q) {
    if (above < s.k_rem && s.k_rem <= above + c[q]) {  // exactly one bin of one thread satisfies this
      GroupState o = s;
      o.prefix = s.prefix | ((uint32_t)(tid * kPer + q) << shift);
      o.k_rem = s.k_rem - above;
      if (last) {
        o.t_key = o.prefix;
        o.need = o.k_rem;
      }
      st[grp] = o;
    }
    above += c[q];
  }
}

// per wave chunk: elements above the threshold key and elements equal to it
template <typename BitsT>
__global__ __launch_bounds__(256) void gsel_count_kernel(const BitsT* __restrict__ A, int64_t n, int64_t g,
                                                         int64_t chunks_per_group, int64_t n_chunks,
                                                         const GroupState* __restrict__ st,
                                                         uint2* __restrict__ ccount) {
  const int lane = threadIdx.x & 63;
  const int64_t id = (int64_t)blockIdx.x * 4 + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  if (id >= n_chunks) return;
  const int64_t grp = id / chunks_per_group, chunk = id % chunks_per_group;
  const int64_t gstart = grp * g;
  const int64_t gend = min(gstart + g, n);
  const int64_t e0 = gstart + chunk * kGlobalWaveChunk;
  const uint32_t t_key = st[grp].t_key;
  uint32_t gt = 0, eq = 0;  // per-lane counts
  constexpr int kBatch = 8;
  for (int r0 = 0; r0 < kGlobalWaveChunk / 64; r0 += kBatch) {
    uint32_t key[kBatch];
    bool valid[kBatch];
#pragma unroll
    for (int q = 0; q < kBatch; ++q) {
      const int64_t e = e0 + (r0 + q) * 64 + lane;
      valid[q] = e < gend;
      key[q] = (uint32_t)A[valid[q] ? e : gend - 1] & Key<BitsT>::kMask;
    }
#pragma unroll
    for (int q = 0; q < kBatch; ++q) {
      gt += (valid[q] && key[q] > t_key) ? 1u : 0u;
      eq += (valid[q] && key[q] == t_key) ? 1u : 0u;
    }
  }
  gt = wave_sum_u32(gt);
  eq = wave_sum_u32(eq);
  if (lane == 0) ccount[id] = make_uint2(gt, eq);
}

// ---------------------------------------------------------------------------------------------------------
// path 4: long groups in two reads of the activation (groups of at least kTwoReadMinGroup elements)
// ---------------------------------------------------------------------------------------------------------
// The radix select of path 3 reads the activation once per digit pass, then once to count and once to pack.  Here a
// sample brackets the threshold first: one workgroup per group draws 2048 elements at hashed positions and takes two
// of the sample's order statistics, `margin` standard deviations of the sample rank to either side of rank k * 2048 /
// len, as the bracket lo_key <= threshold <= hi_key.  One pass over the activation then counts, per 4096-element chunk,
// the elements above the bracket, at its two ends, and strictly inside it, and copies the keys strictly inside (the
// candidates, a few per cent of the group) to the chunk's slot of a side buffer.  The exact threshold is then selected
// among the candidates alone (the digit passes of path 3 over the side buffer, on key - lo_key - 1, whose range the
// bracket makes narrow), the per-chunk counts follow from the chunk's record and slot, and the pack pass of path 3 is
// the second read.  The bracket's ends are counted, not copied: a plateau of equal keys (the zeros behind a ReLU, a
// clipped maximum) sits at an end, where it costs nothing, because both order statistics of the sample fall on it.
// Whether the bracket holds the threshold is known only on the device, after the first pass.  If it does not (a
// sample that far off is a once-in-millions event at the default margin of five deviations), or a chunk has more
// candidates than its slot, the same kernels select over the activation itself: the result is the same, three more
// reads are spent.  Nothing is decided by floating point except which keys are copied.
constexpr int kTwoReadSample = 32;       // sample size / 64: 2048 elements (a larger sample narrows the bracket, but its
                                         // scattered loads, issued by one compute unit, are what the bracketing kernel waits for)
constexpr int kTwoReadSlot = kTwoReadSlotKeys;  // candidate keys a chunk's slot holds


struct Sel2 {  // per group
  uint32_t lo_key, hi_key;  // bracket on the magnitude key; candidates are lo_key < key < hi_key
  uint32_t mode;            // after the decision: 0 = threshold known, 1 = select among the candidates, 2 = over A
  uint32_t base;            // digits are taken from key - base
  uint32_t bits;            // significant bits of the largest key - base
  uint32_t pad[3];
};
struct ChunkRec {
  uint32_t above, top, bottom, cand;  // keys > hi_key, == hi_key, == lo_key (when lo_key != hi_key), strictly inside
};
static_assert(sizeof(Sel2) == 32 && sizeof(ChunkRec) == 16, "the workspace query sizes these");

__device__ __forceinline__ uint32_t mix32(uint32_t x) {
  x ^= x >> 16; x *= 0x85ebca6bu; x ^= x >> 13; x *= 0xc2b2ae35u; x ^= x >> 16;
  return x;
}

// One workgroup of eight wavefronts per group brackets the threshold: wavefronts 0-3 search the upper end, 4-7 the lower
// end, each holding a quarter of the sample (both halves draw the same sample).  A search keeps
// count(key >= lo) >= rank > count(key >= hi) over the sample and probes between them (the in-register selection's
// search: first 16 octaves below the largest key, then key 1, then regula falsi with the Illinois rule); the four
// wavefronts of a search hold identical copies of its state and exchange their part counts through LDS, one barrier
// per probe.  After at most kBracketProbes probes the upper end takes hi - 1 and the lower end lo: both err outwards,
// so a search that has not converged widens the bracket, never invalidates it.  Meanwhile the workgroup clears the
// group's digit histograms (the workspace comes with arbitrary contents).
constexpr int kBracketProbes = 48;
template <typename BitsT>
__global__ __launch_bounds__(512) void sel2_bracket_kernel(const BitsT* __restrict__ A, int64_t n, int64_t g, int64_t n_groups,
                                                           uint32_t k_full, uint32_t k_last, float margin,
                                                           Sel2* __restrict__ sel, uint32_t* __restrict__ hist, int replicas) {
  constexpr int S = kTwoReadSample * 64;
  constexpr int E = kTwoReadSample / 4;  // slots per wavefront
  __shared__ uint32_t part[2][2][4];     // [probe parity][search][wavefront of the search]: part counts
  __shared__ uint32_t live[2][2];        // [probe parity][search]: the search still probes
  __shared__ uint32_t wmax[4];
  __shared__ uint32_t ends[2];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int search = wave >> 2, quarter = wave & 3;
  const int64_t grp = blockIdx.x;
  const int64_t gstart = grp * g;
  const uint32_t len = (uint32_t)(min(gstart + g, n) - gstart);
  const uint32_t k = grp == n_groups - 1 ? k_last : k_full;
  uint32_t kr[E];
#pragma unroll
  for (int j = 0; j < E; ++j) {
    const uint32_t h = mix32((uint32_t)((quarter * E + j) * 64 + lane) * 0x9e3779b9u + 0x7f4a7c15u);
    const uint32_t pos = (uint32_t)(((uint64_t)h * (uint64_t)len) >> 32);
    kr[j] = Key<BitsT>::rot(A[gstart + pos]);
  }
  uint4* __restrict__ hz = reinterpret_cast<uint4*>(hist + grp * replicas * (int64_t)kGlobalHistBins);
  for (int i = threadIdx.x; i < replicas * kGlobalHistBins / 4; i += 512) hz[i] = make_uint4(0u, 0u, 0u, 0u);
  uint32_t m = 0;
#pragma unroll
  for (int j = 0; j < E; ++j) m = max(m, kr[j]);
  m = wave_max_u32(m);
  if (search == 0 && lane == 0) wmax[quarter] = m;
  __syncthreads();
  m = max(max(wmax[0], wmax[1]), max(wmax[2], wmax[3]));

  const float f = (float)k / (float)len;
  const float ks = f * (float)S;
  const float dev = margin * sqrtf((float)S * f * (1.0f - f)) + 2.0f;
  // a rank outside the sample: that end of the bracket is open (0x80000000 is above every key; below, key 0 is the end)
  const int want = search == 0 ? (int)floorf(ks - dev) : (int)ceilf(ks + dev);
  const bool open_end = search == 0 ? want < 1 : want > S;
  const int rank = min(max(want, 1), S);
  uint32_t lo = 0, hi = (m >> 1) + 1;
  float f_lo = (float)(S - rank), f_hi = (float)(-rank);
  int last_side = 0;
  bool tried_one = false, found = false;
  constexpr uint32_t kSixteenOctaves = 16u << (Key<BitsT>::kBits - 8);
  for (int probe = 0; probe < kBracketProbes; ++probe) {
    const int par = probe & 1;
    const bool active = !open_end && !found && hi - lo > 1;
    uint32_t mid = lo;
    if (active) {
      const uint32_t span = hi - lo;
      if (probe == 0 && hi > kSixteenOctaves + 1u) {
        mid = hi - 1u - kSixteenOctaves;
      } else if (lo == 0 && !tried_one) {
        mid = 1;
        tried_one = true;
      } else {
        uint32_t d = (uint32_t)(f_lo * __builtin_amdgcn_rcpf(f_lo - f_hi) * (float)span);
        d = min(max(d, 1u), span - 1u);
        mid = lo + d;
      }
      const int c_part = count_ge<E>(kr, mid << 1);
      if (lane == 0) part[par][search][quarter] = (uint32_t)c_part;
    }
    if (lane == 0 && quarter == 0) live[par][search] = active ? 1u : 0u;
    __syncthreads();
    if (!live[par][0] && !live[par][1]) break;  // the same two words for every wavefront
    if (active) {
      const int c = (int)(part[par][search][0] + part[par][search][1] + part[par][search][2] + part[par][search][3]);
      if (c == rank) {  // not a key of the sample, but as good a bracket end as one
        found = true;
        lo = mid;
        hi = mid + 1;
      } else if (c > rank) {
        lo = mid;
        f_lo = (float)(c - rank);
        if (last_side > 0) f_hi *= 0.5f;
        last_side = 1;
      } else {
        hi = mid;
        f_hi = (float)(c - rank);
        if (last_side < 0) f_lo *= 0.5f;
        last_side = -1;
      }
    }
  }
  if (lane == 0 && quarter == 0) ends[search] = open_end ? (search == 0 ? 0x80000000u : 0u) : (search == 0 ? hi - 1u : lo);
  __syncthreads();
  if (threadIdx.x == 0) {
    Sel2 o;
    o.lo_key = ends[1];
    o.hi_key = max(ends[0], ends[1]);  // a negative margin crosses the ranks: a one-key bracket, decided like any other
    o.mode = 0; o.base = 0; o.bits = 0; o.pad[0] = o.pad[1] = o.pad[2] = 0;
    sel[grp] = o;
  }
}

// first read: per wave chunk the record of counts and the candidate keys.  The four counts come from four nested
// "greater" predicates (their differences), each one compare and one add-with-carry per element.
template <typename BitsT, bool FULL>
__device__ __forceinline__ void sel2_collect_chunk(const BitsT* __restrict__ src, int left, uint32_t lo, uint32_t hi,
                                                   ChunkRec* __restrict__ rec_out, uint32_t* __restrict__ dst) {
  const int lane = threadIdx.x & 63;
  constexpr int kRows = kGlobalWaveChunk / 64;
  uint32_t key[kRows];
  // rows past the end of the group read its last element and are turned into key 0xffffffff, which no count sees
#pragma unroll
  for (int q = 0; q < kRows; ++q) key[q] = (uint32_t)src[FULL ? q * 64 + lane : min(q * 64 + lane, left - 1)];
#pragma unroll
  for (int q = 0; q < kRows; ++q) {
    key[q] &= Key<BitsT>::kMask;
    if (!FULL) key[q] = q * 64 + lane < left ? key[q] : 0xffffffffu;
  }
  // c_gt_hi <= c_ge_hi <= c_gt_lo <= c_ge_lo over the valid keys; an invalid key counts in all four and is taken out below
  uint32_t c_gt_hi = 0, c_ge_hi = 0, c_gt_lo = 0, c_ge_lo = 0;
#pragma unroll
  for (int q = 0; q < kRows; ++q) {
    c_gt_hi += key[q] > hi ? 1u : 0u;
    c_ge_hi += key[q] >= hi ? 1u : 0u;
    c_gt_lo += key[q] > lo ? 1u : 0u;
    c_ge_lo += key[q] >= lo ? 1u : 0u;
  }
  const uint32_t invalid = FULL ? 0u : (uint32_t)(kGlobalWaveChunk - left);
  c_gt_hi = wave_sum_u32(c_gt_hi) - invalid;
  c_ge_hi = wave_sum_u32(c_ge_hi) - invalid;
  c_gt_lo = wave_sum_u32(c_gt_lo) - invalid;
  c_ge_lo = wave_sum_u32(c_ge_lo) - invalid;
  const bool one_key = lo == hi;  // then everything equal to it is `top`, and nothing is inside
  const uint32_t n_cand = one_key ? 0u : c_gt_lo - c_ge_hi;
  if (lane == 0) {
    ChunkRec o;
    o.above = c_gt_hi; o.top = c_ge_hi - c_gt_hi; o.bottom = one_key ? 0u : c_ge_lo - c_gt_lo;
    o.cand = n_cand;  // more than kTwoReadSlot: the slot is not written
    *rec_out = o;
  }
  if (n_cand == 0 || n_cand > (uint32_t)kTwoReadSlot) return;
  uint32_t run = 0;
#pragma unroll
  for (int q = 0; q < kRows; ++q) {
    const bool c = key[q] > lo && key[q] < hi;
    const uint64_t b = ballot64(c);
    if (c) dst[lane_rank(b, run)] = key[q];
    run += (uint32_t)__popcll(b);
  }
}

template <typename BitsT>
__global__ __launch_bounds__(256) void sel2_collect_kernel(const BitsT* __restrict__ A, int64_t n, int64_t g,
                                                           int64_t chunks_per_group, int64_t n_chunks,
                                                           const Sel2* __restrict__ sel, ChunkRec* __restrict__ rec,
                                                           uint32_t* __restrict__ cand) {
  const int64_t id = (int64_t)blockIdx.x * 4 + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  if (id >= n_chunks) return;
  const int64_t grp = id / chunks_per_group, chunk = id % chunks_per_group;
  const int64_t gstart = grp * g;
  const int64_t gend = min(gstart + g, n);
  const int64_t e0 = gstart + chunk * kGlobalWaveChunk;
  const uint32_t lo = sel[grp].lo_key, hi = sel[grp].hi_key;
  const int64_t left = gend - e0;
  if (left <= 0) {  // the last group is shorter than the others and does not reach this chunk
    if ((threadIdx.x & 63) == 0) {
      ChunkRec o;
      o.above = o.top = o.bottom = o.cand = 0;
      rec[id] = o;
    }
    return;
  }
  if (left >= kGlobalWaveChunk)
    sel2_collect_chunk<BitsT, true>(A + e0, kGlobalWaveChunk, lo, hi, rec + id, cand + id * kTwoReadSlot);
  else
    sel2_collect_chunk<BitsT, false>(A + e0, (int)left, lo, hi, rec + id, cand + id * kTwoReadSlot);
}

// Per group: where the threshold lies relative to the bracket, from the sums of the chunk records.
__global__ __launch_bounds__(1024) void sel2_decide_kernel(Sel2* __restrict__ sel, GroupState* __restrict__ st,
                                                           const ChunkRec* __restrict__ rec, int64_t chunks_per_group,
                                                           int64_t n_groups, uint32_t k_full, uint32_t k_last,
                                                           uint32_t key_bits) {
  __shared__ uint32_t tot[5];
  const int64_t grp = blockIdx.x;
  const uint4* __restrict__ r = reinterpret_cast<const uint4*>(rec + grp * chunks_per_group);
  if (threadIdx.x < 5) tot[threadIdx.x] = 0;
  __syncthreads();
  uint32_t above = 0, top = 0, bottom = 0, cnd = 0, over = 0;
  for (int64_t c = threadIdx.x; c < chunks_per_group; c += 1024) {
    const uint4 x = r[c];  // (above, top, bottom, cand)
    above += x.x; top += x.y; bottom += x.z; cnd += x.w;
    over += x.w > (uint32_t)kTwoReadSlot ? 1u : 0u;
  }
  above = wave_sum_u32(above); top = wave_sum_u32(top); bottom = wave_sum_u32(bottom); cnd = wave_sum_u32(cnd);
  over = wave_sum_u32(over);
  if ((threadIdx.x & 63) == 0) {  // integer sums: the order of the atomics does not matter
    atomicAdd(&tot[0], above); atomicAdd(&tot[1], top); atomicAdd(&tot[2], bottom); atomicAdd(&tot[3], cnd);
    atomicAdd(&tot[4], over);
  }
  __syncthreads();
  const uint32_t t_above = tot[0], t_top = tot[1], t_bottom = tot[2], t_cand = tot[3], t_over = tot[4];
  if (threadIdx.x != 0) return;
  const uint32_t k = grp == n_groups - 1 ? k_last : k_full;
  Sel2 s = sel[grp];
  GroupState o;
  o.prefix = 0; o.k_rem = k; o.t_key = 0; o.need = 0;
  s.mode = 2; s.base = 0; s.bits = key_bits;  // unless the bracket holds the threshold: select over A, all key bits
  if (t_over == 0 && k > t_above) {
    uint32_t kk = k - t_above;
    if (kk <= t_top) {
      s.mode = 0; o.t_key = s.hi_key; o.need = kk;
    } else if (kk - t_top <= t_cand) {
      kk -= t_top;
      // largest candidate key - base; an open upper end stands above every key of this dtype (candidates exist, so >= 0)
      const uint32_t vmax = min(s.hi_key, 1u << key_bits) - s.lo_key - 2u;
      s.base = s.lo_key + 1u;
      s.bits = vmax == 0u ? 0u : 32u - (uint32_t)__clz((int)vmax);
      o.k_rem = kk;
      if (s.bits == 0u) {  // one candidate key
        s.mode = 0; o.t_key = s.base; o.need = kk;
      } else {
        s.mode = 1;
      }
    } else if (kk - t_top - t_cand <= t_bottom) {
      s.mode = 0; o.t_key = s.lo_key; o.need = kk - t_top - t_cand;
    }
  }
  sel[grp] = s;
  st[grp] = o;
}

// digit pass `pass` of a group with `bits` significant bits: the bits [shift, shift + nbits) of key - base
__device__ __forceinline__ bool sel2_pass_geometry(uint32_t bits, int pass, int* shift, int* nbits) {
  const int done = kGlobalDigitBits * pass;
  if ((int)bits <= done) return false;
  *shift = max((int)bits - done - kGlobalDigitBits, 0);
  *nbits = (int)bits - done - *shift;
  return true;
}

template <typename BitsT>
__global__ __launch_bounds__(256) void sel2_hist_kernel(const BitsT* __restrict__ A, int64_t n, int64_t g,
                                                        int64_t blocks_per_group, int64_t chunks_per_group, int pass,
                                                        const Sel2* __restrict__ sel, const GroupState* __restrict__ st,
                                                        const ChunkRec* __restrict__ rec, const uint32_t* __restrict__ cand,
                                                        uint32_t* __restrict__ hist, int replicas) {
  __shared__ uint32_t lh[kGlobalHistBins];
  const int64_t grp = blockIdx.x / blocks_per_group;
  const int64_t blk = blockIdx.x % blocks_per_group;
  const Sel2 s = sel[grp];
  int shift, nbits;
  if (s.mode == 0 || !sel2_pass_geometry(s.bits, pass, &shift, &nbits)) return;
  for (int b = threadIdx.x; b < kGlobalHistBins; b += 256) lh[b] = 0;
  __syncthreads();
  const int hshift = shift + nbits;  // <= 31
  const uint32_t want = st[grp].prefix >> hshift;
  const uint32_t dmask = (1u << nbits) - 1u;
  const int lane = threadIdx.x & 63;
  uint32_t zeros = 0;  // elements of this wavefront with digit 0 (wave-uniform): one ballot instead of same-address atomics
  if (s.mode == 2) {
    const int64_t gstart = grp * g;
    const int64_t gend = min(gstart + g, n);
    const int64_t e0 = gstart + blk * kGlobalHistChunk;
    constexpr int kBatch = 8;
    for (int t0 = 0; t0 < kGlobalHistChunk; t0 += 256 * kBatch) {
      uint32_t key[kBatch];
      bool ok[kBatch];
#pragma unroll
      for (int q = 0; q < kBatch; ++q) {
        const int64_t e = e0 + t0 + q * 256 + threadIdx.x;
        ok[q] = e < gend;
        key[q] = (uint32_t)A[ok[q] ? e : gend - 1] & Key<BitsT>::kMask;
      }
#pragma unroll
      for (int q = 0; q < kBatch; ++q) {
        const bool match = ok[q] && (key[q] >> hshift) == want;
        const uint32_t digit = (key[q] >> shift) & dmask;
        zeros += (uint32_t)__popcll(ballot64(match && digit == 0u));
        if (match && digit != 0u) atomicAdd(&lh[digit], 1u);
      }
    }
  } else {
    // one chunk's slot per wavefront (kGlobalHistChunk / kGlobalWaveChunk = 4 = the wavefronts of the workgroup)
    static_assert(kGlobalHistChunk / kGlobalWaveChunk == 4, "one slot per wavefront");
    const int64_t chunk = blk * 4 + (threadIdx.x >> 6);
    if (chunk < chunks_per_group) {
      const int64_t id = grp * chunks_per_group + chunk;
      const uint32_t cnt = rec[id].cand;  // <= kTwoReadSlot in this mode
      const uint32_t* __restrict__ src = cand + id * kTwoReadSlot;
      for (uint32_t i0 = 0; i0 < cnt; i0 += 64) {  // wave-uniform trip count: the ballot below needs the whole wavefront
        const uint32_t i = i0 + lane;
        const bool ok = i < cnt;
        const uint32_t v = (ok ? src[i] : s.base) - s.base;
        const bool match = ok && (v >> hshift) == want;
        const uint32_t digit = (v >> shift) & dmask;
        zeros += (uint32_t)__popcll(ballot64(match && digit == 0u));
        if (match && digit != 0u) atomicAdd(&lh[digit], 1u);
      }
    }
  }
  if (lane == 0 && zeros) atomicAdd(&lh[0], zeros);
  __syncthreads();
  uint32_t* __restrict__ h = hist + (grp * replicas + blk % replicas) * (int64_t)kGlobalHistBins;
  for (int b = threadIdx.x; b < kGlobalHistBins; b += 256) {
    const uint32_t c = lh[b];
    if (c) atomicAdd(&h[b], c);
  }
}

// Picks the digit that holds the k_rem-th largest matching element of each group and clears its histograms for the next
// pass.  (A separate launch on purpose: letting the group's last histogram workgroup do this needs a device-scope
// fence in every workgroup, which on this chip costs far more than the launch: 59 against 6 + 5 microseconds.)
__global__ __launch_bounds__(256) void sel2_resolve_kernel(const Sel2* __restrict__ sel, GroupState* __restrict__ st,
                                                           uint32_t* __restrict__ hist, int replicas, int pass) {
  constexpr int kPer = kGlobalHistBins / 256;
  static_assert(kPer % 4 == 0, "16-byte loads");
  __shared__ uint32_t lds17[17];
  const int64_t grp = blockIdx.x;
  const Sel2 sl = sel[grp];
  int shift, nbits;
  if (sl.mode == 0 || !sel2_pass_geometry(sl.bits, pass, &shift, &nbits)) return;  // its histogram was not touched
  const int tid = threadIdx.x;
  uint32_t* __restrict__ h = hist + grp * replicas * (int64_t)kGlobalHistBins;
  uint32_t c[kPer];
  uint32_t sum = 0;
#pragma unroll
  for (int q = 0; q < kPer; ++q) c[q] = 0;
  for (int rep = 0; rep < replicas; ++rep) {  // all loads before the first store: they do not wait for each other
    const uint4* __restrict__ src = reinterpret_cast<const uint4*>(h + rep * kGlobalHistBins + tid * kPer);
#pragma unroll
    for (int q = 0; q < kPer; q += 4) {
      const uint4 x = src[q / 4];
      c[q] += x.x; c[q + 1] += x.y; c[q + 2] += x.z; c[q + 3] += x.w;
    }
  }
  for (int rep = 0; rep < replicas; ++rep) {
    uint4* __restrict__ dst = reinterpret_cast<uint4*>(h + rep * kGlobalHistBins + tid * kPer);
#pragma unroll
    for (int q = 0; q < kPer; q += 4) dst[q / 4] = make_uint4(0u, 0u, 0u, 0u);
  }
#pragma unroll
  for (int q = 0; q < kPer; ++q) sum += c[q];
  const GroupState s = st[grp];
  uint32_t total;
  const uint32_t below = block_excl_scan(sum, lds17, &total);
  uint32_t above = total - below - sum;
#pragma unroll
  for (int q = kPer - 1; q >= 0; --q) {
    if (above < s.k_rem && s.k_rem <= above + c[q]) {  // exactly one bin of one thread satisfies this
      GroupState o = s;
      o.prefix = s.prefix | ((uint32_t)(tid * kPer + q) << shift);
      o.k_rem = s.k_rem - above;
      if (shift == 0) {
        o.t_key = sl.base + o.prefix;
        o.need = o.k_rem;
      }
      st[grp] = o;
    }
    above += c[q];
  }
}

// per wave chunk: elements above the threshold key and elements equal to it, from the chunk's record and slot
template <typename BitsT>
__global__ __launch_bounds__(256) void sel2_count_kernel(const BitsT* __restrict__ A, int64_t n, int64_t g,
                                                         int64_t chunks_per_group, int64_t n_chunks,
                                                         const Sel2* __restrict__ sel, const GroupState* __restrict__ st,
                                                         const ChunkRec* __restrict__ rec, const uint32_t* __restrict__ cand,
                                                         uint2* __restrict__ ccount) {
  const int lane = threadIdx.x & 63;
  const int64_t id = (int64_t)blockIdx.x * 4 + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  if (id >= n_chunks) return;
  const int64_t grp = id / chunks_per_group, chunk = id % chunks_per_group;
  const Sel2 s = sel[grp];
  const uint32_t t_key = st[grp].t_key;
  uint32_t gt = 0, eq = 0;  // per-lane counts
  if (s.mode == 2) {
    const int64_t gstart = grp * g;
    const int64_t gend = min(gstart + g, n);
    const int64_t e0 = gstart + chunk * kGlobalWaveChunk;
    constexpr int kBatch = 8;
    for (int r0 = 0; r0 < kGlobalWaveChunk / 64; r0 += kBatch) {
      uint32_t key[kBatch];
      bool valid[kBatch];
#pragma unroll
      for (int q = 0; q < kBatch; ++q) {
        const int64_t e = e0 + (r0 + q) * 64 + lane;
        valid[q] = e < gend;
        key[q] = (uint32_t)A[valid[q] ? e : gend - 1] & Key<BitsT>::kMask;
      }
#pragma unroll
      for (int q = 0; q < kBatch; ++q) {
        gt += (valid[q] && key[q] > t_key) ? 1u : 0u;
        eq += (valid[q] && key[q] == t_key) ? 1u : 0u;
      }
    }
    gt = wave_sum_u32(gt);
    eq = wave_sum_u32(eq);
  } else {
    const ChunkRec x = rec[id];
    const uint32_t* __restrict__ src = cand + id * kTwoReadSlot;
    for (uint32_t i = lane; i < x.cand; i += 64) {
      const uint32_t key = src[i];
      gt += key > t_key ? 1u : 0u;
      eq += key == t_key ? 1u : 0u;
    }
    gt = wave_sum_u32(gt) + x.above + (s.hi_key > t_key ? x.top : 0u);
    eq = wave_sum_u32(eq) + (s.hi_key == t_key ? x.top : 0u) + (s.lo_key == t_key ? x.bottom : 0u);
  }
  if (lane == 0) ccount[id] = make_uint2(gt, eq);
}

// Per group: exclusive prefix over its chunks of (equal elements seen, values written).  One workgroup of 1024
// threads; a thread holds kScanPer consecutive chunks in registers, so a tile of 1024 * kScanPer chunks costs one
// round of loads, two block-wide scans (ties first: how many tied elements a chunk may keep depends on the ties
// before it) and one round of stores.
constexpr int kScanPer = 8;
__global__ __launch_bounds__(1024) void gsel_scan_kernel(const GroupState* __restrict__ st,
                                                         const uint2* __restrict__ ccount, uint2* __restrict__ cbase,
                                                         int64_t chunks_per_group) {
  __shared__ uint32_t lds17[17];
  const int64_t grp = blockIdx.x;
  const uint2* __restrict__ cc = ccount + grp * chunks_per_group;
  uint2* __restrict__ cb = cbase + grp * chunks_per_group;
  const uint32_t need = st[grp].need;
  uint32_t eq_carry = 0, out_carry = 0;
  for (int64_t tile0 = 0; tile0 < chunks_per_group; tile0 += 1024 * kScanPer) {
    const int64_t c0 = tile0 + (int64_t)threadIdx.x * kScanPer;
    uint2 v[kScanPer];
    uint32_t eq_sum = 0;
#pragma unroll
    for (int q = 0; q < kScanPer; ++q) {
      v[q] = c0 + q < chunks_per_group ? cc[c0 + q] : make_uint2(0u, 0u);
      eq_sum += v[q].y;
    }
    uint32_t eq_total, out_total;
    uint32_t eq_before = eq_carry + block_excl_scan(eq_sum, lds17, &eq_total);
    uint32_t eqb[kScanPer], kept_sum = 0;
#pragma unroll
    for (int q = 0; q < kScanPer; ++q) {
      eqb[q] = eq_before;
      const uint32_t take = eq_before >= need ? 0u : min(need - eq_before, v[q].y);
      v[q].x += take;  // values this chunk writes
      kept_sum += v[q].x;
      eq_before += v[q].y;
    }
    uint32_t out_before = out_carry + block_excl_scan(kept_sum, lds17, &out_total);
#pragma unroll
    for (int q = 0; q < kScanPer; ++q) {
      if (c0 + q < chunks_per_group) cb[c0 + q] = make_uint2(eqb[q], out_before);
      out_before += v[q].x;
    }
    eq_carry += eq_total;
    out_carry += out_total;
  }
}

// DIRECT: every group starts on a mask word, so a row of 64 elements is one whole word, stored as such; otherwise the
// rows are OR-ed into a zeroed mask.
template <typename BitsT, bool WITH_IDX, bool DIRECT>
__global__ __launch_bounds__(256) void gsel_pack_kernel(const BitsT* __restrict__ A, int64_t n, int64_t g,
                                                        int64_t chunks_per_group, int64_t n_chunks,
                                                        const GroupState* __restrict__ st,
                                                        const uint2* __restrict__ cbase, int64_t k_full,
                                                        BitsT* __restrict__ vals, uint64_t* __restrict__ mask,
                                                        uint32_t* __restrict__ idx) {
  const int lane = threadIdx.x & 63;
  const int64_t id = (int64_t)blockIdx.x * 4 + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  if (id >= n_chunks) return;
  const int64_t grp = id / chunks_per_group, chunk = id % chunks_per_group;
  const int64_t gstart = grp * g;
  const int64_t gend = min(gstart + g, n);
  const int64_t e0 = gstart + chunk * kGlobalWaveChunk;
  const GroupState s = st[grp];
  const uint2 base = cbase[id];
  uint32_t eq_run = base.x, run = base.y;
  BitsT* __restrict__ out_vals = vals + grp * k_full;
  uint32_t* __restrict__ out_idx = WITH_IDX ? idx + grp * k_full : nullptr;
  constexpr int kBatch = 8;  // rows of 64 elements requested together
  for (int r0 = 0; r0 < kGlobalWaveChunk / 64; r0 += kBatch) {
    if (e0 + r0 * 64 >= gend) break;
    BitsT row[kBatch];
#pragma unroll
    for (int q = 0; q < kBatch; ++q) {
      const int64_t e = e0 + (r0 + q) * 64 + lane;
      row[q] = A[e < gend ? e : gend - 1];
    }
#pragma unroll
    for (int q = 0; q < kBatch; ++q) {
      const int64_t e_first = e0 + (r0 + q) * 64;
      if (e_first < gend) {
        const int64_t e = e_first + lane;
        const bool valid = e < gend;
        const BitsT bits = row[q];
        const uint32_t key = (uint32_t)bits & Key<BitsT>::kMask;
        const bool gt = valid && key > s.t_key;
        const bool eq = valid && key == s.t_key;
        const uint64_t beq = ballot64(eq);
        const bool keep = gt || (eq && lane_rank(beq, eq_run) < s.need);
        const uint64_t b = ballot64(keep);
        if (keep) {
          const uint32_t o = lane_rank(b, run);
          out_vals[o] = bits;
          if (WITH_IDX) out_idx[o] = (uint32_t)(e - gstart);
        }
        if constexpr (DIRECT) {
          if (lane == 0) mask[e_first >> 6] = b;
        } else {
          or_into_mask(mask, e_first, b, lane);
        }
        run += (uint32_t)__popcll(b);
        eq_run += (uint32_t)__popcll(beq);
      }
    }
  }
}

template <typename BitsT>
static int launch_gsel_pack(const GroupPlan& p, int64_t cpg, int64_t n_chunks, const void* A, const GroupState* state,
                            const uint2* cbase, void* vals, uint64_t* mask, uint32_t* idx, bool direct, hipStream_t st) {
  const dim3 wgrid((unsigned)ceil_div(n_chunks, 4)), block(256);
#define SURGEON_PACK(IDX, DIR)                                                                                        \
  SURGEON_LAUNCH((gsel_pack_kernel<BitsT, IDX, DIR>), wgrid, block, 0, st, (const BitsT*)A, p.n, p.g, cpg, n_chunks, \
                     state, cbase, p.k_full, (BitsT*)vals, mask, idx)
  if (idx && direct) SURGEON_PACK(true, true);
  else if (idx) SURGEON_PACK(true, false);
  else if (direct) SURGEON_PACK(false, true);
  else SURGEON_PACK(false, false);
#undef SURGEON_PACK
  SURGEON_LAUNCH_CHECK();
  return SURGEON_OK;
}

// groups that start on mask words: the pack pass of the long-group paths then stores whole words and needs no zeroed mask
static bool groups_word_aligned(const GroupPlan& p) { return p.n_groups == 1 || p.g % 64 == 0; }

// ---------------------------------------------------------------------------------------------------------
// host dispatch
// ---------------------------------------------------------------------------------------------------------
static int zero_mask(uint64_t* mask, int64_t n_words, hipStream_t st) {
  if (n_words == 0) return SURGEON_OK;
  const int blocks = (int)std::min<int64_t>(ceil_div(n_words, 256), 4096);
  SURGEON_LAUNCH(fill_zero_u64_kernel, dim3(blocks), dim3(256), 0, st, mask, n_words);
  SURGEON_LAUNCH_CHECK();
  return SURGEON_OK;
}

template <int E, typename BitsT>
static int launch_wave_reg(const GroupPlan& p, const void* A, void* vals, uint64_t* mask, uint32_t* idx,
                           hipStream_t st) {
  const dim3 grid((unsigned)ceil_div(p.n_groups, 4)), block(256);
  ProfScope prof(SURGEON_PROF_SELECT_PACK, st);
  if (idx)
    SURGEON_LAUNCH((select_pack_wave_reg_kernel<E, BitsT, true>), grid, block, 0, st, (const BitsT*)A, (BitsT*)vals,
                       mask, idx, p.n_groups, (int)p.g, (int)p.len_last, (int)p.k_full, (int)p.k_last);
  else
    SURGEON_LAUNCH((select_pack_wave_reg_kernel<E, BitsT, false>), grid, block, 0, st, (const BitsT*)A,
                       (BitsT*)vals, mask, idx, p.n_groups, (int)p.g, (int)p.len_last, (int)p.k_full, (int)p.k_last);
  SURGEON_LAUNCH_CHECK();
  return SURGEON_OK;
}

template <typename BitsT>
static int run_wave_reg(const GroupPlan& p, const void* A, void* vals, uint64_t* mask, uint32_t* idx, hipStream_t st) {
  const int slots = (int)(p.g / 64);
  if (slots <= 1) return launch_wave_reg<1, BitsT>(p, A, vals, mask, idx, st);
  if (slots <= 2) return launch_wave_reg<2, BitsT>(p, A, vals, mask, idx, st);
  if (slots <= 4) return launch_wave_reg<4, BitsT>(p, A, vals, mask, idx, st);
  if (slots <= 8) return launch_wave_reg<8, BitsT>(p, A, vals, mask, idx, st);
  if (slots <= 12) return launch_wave_reg<12, BitsT>(p, A, vals, mask, idx, st);
  if (slots <= 16) return launch_wave_reg<16, BitsT>(p, A, vals, mask, idx, st);
  if (slots <= 24) return launch_wave_reg<24, BitsT>(p, A, vals, mask, idx, st);
  if (slots <= 32) return launch_wave_reg<32, BitsT>(p, A, vals, mask, idx, st);
  if (slots <= 48) return launch_wave_reg<48, BitsT>(p, A, vals, mask, idx, st);
  return launch_wave_reg<64, BitsT>(p, A, vals, mask, idx, st);
}

// register slots per lane the in-register kernel is built with for a group length
static int wave_reg_slots(int64_t g) {
  const int slots = (int)(g / 64);
  const int built[10] = {1, 2, 4, 8, 12, 16, 24, 32, 48, 64};
  for (int i = 0; i < 10; ++i)
    if (slots <= built[i]) return built[i];
  return 64;
}

template <int E, typename BitsT>
static int launch_wave_reg_batched(const PackBatch& bt, int blocks, hipStream_t st) {
  ProfScope prof(SURGEON_PROF_SELECT_PACK, st);
  SURGEON_LAUNCH((select_pack_wave_reg_batched_kernel<E, BitsT>), dim3((unsigned)blocks), dim3(256), 0, st, bt);
  SURGEON_LAUNCH_CHECK();
  return SURGEON_OK;
}

template <typename BitsT>
static int run_wave_reg_batched(int slots, const PackBatch& bt, int blocks, hipStream_t st) {
  switch (slots) {
    case 1: return launch_wave_reg_batched<1, BitsT>(bt, blocks, st);
    case 2: return launch_wave_reg_batched<2, BitsT>(bt, blocks, st);
    case 4: return launch_wave_reg_batched<4, BitsT>(bt, blocks, st);
    case 8: return launch_wave_reg_batched<8, BitsT>(bt, blocks, st);
    case 12: return launch_wave_reg_batched<12, BitsT>(bt, blocks, st);
    case 16: return launch_wave_reg_batched<16, BitsT>(bt, blocks, st);
    case 24: return launch_wave_reg_batched<24, BitsT>(bt, blocks, st);
    case 32: return launch_wave_reg_batched<32, BitsT>(bt, blocks, st);
    case 48: return launch_wave_reg_batched<48, BitsT>(bt, blocks, st);
    default: return launch_wave_reg_batched<64, BitsT>(bt, blocks, st);
  }
}

template <typename BitsT>
static int run_wave_mem(const GroupPlan& p, const void* A, void* vals, uint64_t* mask, uint32_t* idx, hipStream_t st) {
  const dim3 grid((unsigned)ceil_div(p.n_groups, 4)), block(256);
  if (idx)
    SURGEON_LAUNCH((select_pack_wave_mem_kernel<BitsT, true>), grid, block, 0, st, (const BitsT*)A, (BitsT*)vals,
                       mask, idx, p.n_groups, (int)p.g, (int)p.len_last, (int)p.k_full, (int)p.k_last);
  else
    SURGEON_LAUNCH((select_pack_wave_mem_kernel<BitsT, false>), grid, block, 0, st, (const BitsT*)A, (BitsT*)vals,
                       mask, idx, p.n_groups, (int)p.g, (int)p.len_last, (int)p.k_full, (int)p.k_last);
  SURGEON_LAUNCH_CHECK();
  return SURGEON_OK;
}

template <typename BitsT>
static int run_global(const GroupPlan& p, const void* A, void* vals, uint64_t* mask, uint32_t* idx, void* ws,
                      hipStream_t st) {
  const int64_t cpg = ceil_div(p.g, kGlobalWaveChunk);
  const int64_t n_chunks = p.n_groups * cpg;
  const int64_t bpg = ceil_div(p.g, kGlobalHistChunk);
  if (p.n_groups * bpg > 0x7fffffffLL || n_chunks > 0x7fffffffLL)
    return fail(SURGEON_EUNSUPPORTED, "prune_pack: too many chunks");
  char* w = (char*)ws;
  GroupState* state = (GroupState*)w;
  w += align_up((size_t)p.n_groups * 16, 256);
  uint32_t* hist = (uint32_t*)w;
  const int replicas = global_hist_replicas(p);
  w += align_up((size_t)p.n_groups * replicas * kGlobalHistBins * 4, 256);
  uint2* ccount = (uint2*)w;
  w += align_up((size_t)n_chunks * 8, 256);
  uint2* cbase = (uint2*)w;

  const int init_blocks = (int)std::min<int64_t>(ceil_div(p.n_groups * replicas * kGlobalHistBins, 256), 4096);
  SURGEON_LAUNCH(gsel_init_kernel, dim3(init_blocks), dim3(256), 0, st, state, hist, p.n_groups,
                     (uint32_t)p.k_full, (uint32_t)p.k_last, replicas);
  SURGEON_LAUNCH_CHECK();
  // digits from the top: 11, 11, 9 bits for the 31-bit fp32 key; 11, 4 for the 15-bit bf16 key
  int shift = Key<BitsT>::kBits;
  while (shift > 0) {
    const int nbits = shift >= kGlobalDigitBits ? kGlobalDigitBits : shift;
    shift -= nbits;
    SURGEON_LAUNCH((gsel_hist_kernel<BitsT>), dim3((unsigned)(p.n_groups * bpg)), dim3(256), 0, st,
                       (const BitsT*)A, p.n, p.g, bpg, shift, nbits, (const GroupState*)state, hist, replicas);
    SURGEON_LAUNCH_CHECK();
    SURGEON_LAUNCH(gsel_resolve_kernel, dim3((unsigned)p.n_groups), dim3(256), 0, st, state, hist, replicas, shift,
                       shift == 0 ? 1 : 0);
    SURGEON_LAUNCH_CHECK();
  }
  const dim3 wgrid((unsigned)ceil_div(n_chunks, 4)), block(256);
  SURGEON_LAUNCH((gsel_count_kernel<BitsT>), wgrid, block, 0, st, (const BitsT*)A, p.n, p.g, cpg, n_chunks,
                     (const GroupState*)state, ccount);
  SURGEON_LAUNCH_CHECK();
  SURGEON_LAUNCH(gsel_scan_kernel, dim3((unsigned)p.n_groups), dim3(1024), 0, st, (const GroupState*)state,
                     (const uint2*)ccount, cbase, cpg);
  SURGEON_LAUNCH_CHECK();
  return launch_gsel_pack<BitsT>(p, cpg, n_chunks, A, (const GroupState*)state, (const uint2*)cbase, vals, mask, idx,
                                 groups_word_aligned(p), st);
}

static std::atomic<float> g_two_read_margin{5.0f};  // read once per call; a plain tuning value, no ordering needed

template <typename BitsT>
static int run_two_read(const GroupPlan& p, const void* A, void* vals, uint64_t* mask, uint32_t* idx, void* ws,
                        hipStream_t st) {
  const int64_t cpg = ceil_div(p.g, kGlobalWaveChunk);
  const int64_t n_chunks = p.n_groups * cpg;
  const int64_t bpg = ceil_div(p.g, kGlobalHistChunk);
  if (p.n_groups * bpg > 0x7fffffffLL || n_chunks > 0x7fffffffLL)
    return fail(SURGEON_EUNSUPPORTED, "prune_pack: too many chunks");
  // the workspace of path 3 first, in its order, then this path's own
  char* w = (char*)ws;
  GroupState* state = (GroupState*)w;
  w += align_up((size_t)p.n_groups * 16, 256);
  uint32_t* hist = (uint32_t*)w;
  const int replicas = global_hist_replicas(p);
  w += align_up((size_t)p.n_groups * replicas * kGlobalHistBins * 4, 256);
  uint2* ccount = (uint2*)w;
  w += align_up((size_t)n_chunks * 8, 256);
  uint2* cbase = (uint2*)w;
  w += align_up((size_t)n_chunks * 8, 256);
  Sel2* sel = (Sel2*)w;
  w += align_up((size_t)p.n_groups * sizeof(Sel2), 256);
  ChunkRec* rec = (ChunkRec*)w;
  w += align_up((size_t)n_chunks * sizeof(ChunkRec), 256);
  uint32_t* cand = (uint32_t*)w;

  SURGEON_LAUNCH((sel2_bracket_kernel<BitsT>), dim3((unsigned)p.n_groups), dim3(512), 0, st, (const BitsT*)A, p.n, p.g,
                     p.n_groups, (uint32_t)p.k_full, (uint32_t)p.k_last, g_two_read_margin.load(std::memory_order_relaxed), sel, hist, replicas);
  SURGEON_LAUNCH_CHECK();
  const dim3 wgrid((unsigned)ceil_div(n_chunks, 4)), block(256);
  SURGEON_LAUNCH((sel2_collect_kernel<BitsT>), wgrid, block, 0, st, (const BitsT*)A, p.n, p.g, cpg, n_chunks,
                     (const Sel2*)sel, rec, cand);
  SURGEON_LAUNCH_CHECK();
  SURGEON_LAUNCH(sel2_decide_kernel, dim3((unsigned)p.n_groups), dim3(1024), 0, st, sel, state, (const ChunkRec*)rec, cpg,
                     p.n_groups, (uint32_t)p.k_full, (uint32_t)p.k_last, (uint32_t)Key<BitsT>::kBits);
  SURGEON_LAUNCH_CHECK();
  // digit passes for all bits of the key (3 for fp32, 2 for bf16): how many a group needs is known only on the
  // device, and a group that needs fewer skips the rest
  const int passes = (Key<BitsT>::kBits + kGlobalDigitBits - 1) / kGlobalDigitBits;
  for (int pass = 0; pass < passes; ++pass) {
    SURGEON_LAUNCH((sel2_hist_kernel<BitsT>), dim3((unsigned)(p.n_groups * bpg)), dim3(256), 0, st, (const BitsT*)A, p.n,
                       p.g, bpg, cpg, pass, (const Sel2*)sel, (const GroupState*)state, (const ChunkRec*)rec,
                       (const uint32_t*)cand, hist, replicas);
    SURGEON_LAUNCH_CHECK();
    SURGEON_LAUNCH(sel2_resolve_kernel, dim3((unsigned)p.n_groups), dim3(256), 0, st, (const Sel2*)sel, state, hist,
                       replicas, pass);
    SURGEON_LAUNCH_CHECK();
  }
  SURGEON_LAUNCH((sel2_count_kernel<BitsT>), wgrid, block, 0, st, (const BitsT*)A, p.n, p.g, cpg, n_chunks,
                     (const Sel2*)sel, (const GroupState*)state, (const ChunkRec*)rec, (const uint32_t*)cand, ccount);
  SURGEON_LAUNCH_CHECK();
  SURGEON_LAUNCH(gsel_scan_kernel, dim3((unsigned)p.n_groups), dim3(1024), 0, st, (const GroupState*)state,
                     (const uint2*)ccount, cbase, cpg);
  SURGEON_LAUNCH_CHECK();
  return launch_gsel_pack<BitsT>(p, cpg, n_chunks, A, (const GroupState*)state, (const uint2*)cbase, vals, mask, idx,
                                 groups_word_aligned(p), st);
}

template <typename BitsT>
static int run_prune_pack(const GroupPlan& p, const void* A, void* vals, uint64_t* mask, uint32_t* idx, void* ws,
                          hipStream_t st) {
  const int64_t n_words = ceil_div(p.n, 64);
  const PrunePath path = choose_prune_path(p);
  if (p.k_total > 0 && path == PATH_WAVE_REG) return run_wave_reg<BitsT>(p, A, vals, mask, idx, st);
  ProfScope prof(SURGEON_PROF_SELECT_OTHER, st);
  if (p.k_total == 0) return zero_mask(mask, n_words, st);
  switch (path) {
    case PATH_WAVE_REG:
      return run_wave_reg<BitsT>(p, A, vals, mask, idx, st);
    case PATH_WAVE_MEM: {
      const int rc = zero_mask(mask, n_words, st);
      if (rc != SURGEON_OK) return rc;
      return run_wave_mem<BitsT>(p, A, vals, mask, idx, st);
    }
    default: {
      const int rc = groups_word_aligned(p) ? SURGEON_OK : zero_mask(mask, n_words, st);
      if (rc != SURGEON_OK) return rc;
      if (path == PATH_TWO_READ) return run_two_read<BitsT>(p, A, vals, mask, idx, ws, st);
      return run_global<BitsT>(p, A, vals, mask, idx, ws, st);
    }
  }
}

}  // namespace surgeon

using namespace surgeon;

extern "C" int surgeon_prune_pack(const void* A, int64_t n, int64_t group_len, float r, int dt, void* vals,
                                  uint64_t* mask, uint32_t* idx, void* ws, size_t ws_bytes, void* stream) {
  if (dt != SURGEON_F32 && dt != SURGEON_BF16) return fail(SURGEON_EINVAL, "prune_pack: bad dtype %d", dt);
  GroupPlan p;
  if (!make_group_plan(n, group_len, r, &p))
    return fail(SURGEON_EINVAL, "prune_pack: need n >= 0, group_len >= 1, 0 <= r <= 1 (n=%lld group_len=%lld r=%g)",
                (long long)n, (long long)group_len, (double)r);
  if (n > ((int64_t)1 << 31)) return fail(SURGEON_EUNSUPPORTED, "prune_pack: n = %lld exceeds 2^31", (long long)n);
  if (n == 0) return SURGEON_OK;
  if (!A || !mask || (p.k_total > 0 && !vals)) return fail(SURGEON_EINVAL, "prune_pack: null pointer");
  const size_t es = dt == SURGEON_F32 ? 4 : 2;
  if (((uintptr_t)A % es) || ((uintptr_t)vals % es) || ((uintptr_t)mask % 8) || ((uintptr_t)idx % 4))
    return fail(SURGEON_EINVAL, "prune_pack: misaligned pointer");
  const size_t need = prune_pack_ws_bytes(p);
  if (need > 0 && (!ws || ws_bytes < need))
    return fail(SURGEON_ESIZE, "prune_pack: workspace of %zu bytes needed, %zu given", need, ws_bytes);
  if (need > 0 && ((uintptr_t)ws % 16)) return fail(SURGEON_EINVAL, "prune_pack: workspace not 16-byte aligned");
  hipStream_t st = (hipStream_t)stream;
  if (dt == SURGEON_F32) return run_prune_pack<uint32_t>(p, A, vals, mask, idx, ws, st);
  return run_prune_pack<uint16_t>(p, A, vals, mask, idx, ws, st);
}

// ---- benchmark aid: the memory pattern of path 1 without its selection ----
template <typename BitsT>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(4))) void select_pack_pattern_probe_kernel(
    const BitsT* __restrict__ A, BitsT* __restrict__ vals, uint64_t* __restrict__ mask, int64_t n_groups, uint32_t thr,
    uint32_t k_cap) {
  constexpr int E = 64;
  const int lane = threadIdx.x & 63;
  const int64_t grp = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (grp >= n_groups) return;
  const BitsT* __restrict__ src = A + grp * (int64_t)(E * 64);
  uint32_t kr[E];
#pragma unroll
  for (int j = 0; j < E; ++j) kr[j] = (uint32_t)src[j * 64 + lane];
  BitsT* __restrict__ dst = vals + grp * (int64_t)k_cap;
  uint32_t base = 0;
  uint64_t word = 0;
#pragma unroll
  for (int j = 0; j < E; ++j) {
    const bool keep = (kr[j] & Key<BitsT>::kMask) >= thr;
    const uint64_t b = ballot64(keep);
    const uint32_t pos = lane_rank(b, base);
    if (keep && pos < k_cap) dst[pos] = (BitsT)kr[j];
    if (lane == j) word = b;
    base += (uint32_t)__popcll(b);
  }
  mask[grp * E + lane] = word;
}

extern "C" int surgeon_select_pack_pattern_probe(const void* A, int64_t n, int dt, uint32_t threshold_bits, int64_t k_cap,
                                                 void* vals, uint64_t* mask, void* stream) {
  if (dt != SURGEON_F32 && dt != SURGEON_BF16) return fail(SURGEON_EINVAL, "pattern probe: bad dtype %d", dt);
  if (n < 0 || n % 4096 || k_cap < 0 || k_cap > 4096) return fail(SURGEON_EINVAL, "pattern probe: n must be a multiple of 4096, k_cap in [0, 4096]");
  if (n == 0) return SURGEON_OK;
  if (!A || !vals || !mask) return fail(SURGEON_EINVAL, "pattern probe: null pointer");
  const int64_t n_groups = n / 4096;
  if (ceil_div(n_groups, 4) > 0x7fffffff) return fail(SURGEON_EUNSUPPORTED, "pattern probe: tensor too large");
  hipStream_t st = (hipStream_t)stream;
  ProfScope prof(SURGEON_PROF_SELECT_OTHER, st);
  const dim3 grid((unsigned)ceil_div(n_groups, 4));
  if (dt == SURGEON_F32)
    SURGEON_LAUNCH(select_pack_pattern_probe_kernel<uint32_t>, grid, dim3(256), 0, st, (const uint32_t*)A, (uint32_t*)vals, mask,
                   n_groups, threshold_bits, (uint32_t)k_cap);
  else
    SURGEON_LAUNCH(select_pack_pattern_probe_kernel<uint16_t>, grid, dim3(256), 0, st, (const uint16_t*)A, (uint16_t*)vals, mask,
                   n_groups, threshold_bits, (uint32_t)k_cap);
  SURGEON_LAUNCH_CHECK();
  return SURGEON_OK;
}

extern "C" int surgeon_set_select_margin(float deviations) {
  if (!(deviations >= -100.0f && deviations <= 100.0f)) return fail(SURGEON_EINVAL, "select margin %g outside [-100, 100]", (double)deviations);
  g_two_read_margin.store(deviations, std::memory_order_relaxed);
  return SURGEON_OK;
}

extern "C" int surgeon_prune_pack_batched(int l, const void* const* A, const int64_t* n, const int64_t* group_len,
                                          const float* r, int dt, void* const* vals, uint64_t* const* mask, void* stream) {
  if (dt != SURGEON_F32 && dt != SURGEON_BF16) return fail(SURGEON_EINVAL, "prune_pack_batched: bad dtype %d", dt);
  if (l < 0 || (l > 0 && (!A || !n || !group_len || !r || !vals || !mask)))
    return fail(SURGEON_EINVAL, "prune_pack_batched: bad arguments");
  const size_t es = dt == SURGEON_F32 ? 4 : 2;
  // validate everything before the first launch
  std::vector<GroupPlan> plans((size_t)l);
  for (int i = 0; i < l; ++i) {
    GroupPlan& p = plans[(size_t)i];
    if (!make_group_plan(n[i], group_len[i], r[i], &p))
      return fail(SURGEON_EINVAL, "prune_pack_batched: tensor %d: need n >= 0, group_len >= 1, 0 <= r <= 1", i);
    if (n[i] > ((int64_t)1 << 31)) return fail(SURGEON_EUNSUPPORTED, "prune_pack_batched: tensor %d exceeds 2^31 elements", i);
    if (n[i] == 0) continue;
    if (choose_prune_path(p) != PATH_WAVE_REG)
      return fail(SURGEON_EUNSUPPORTED,
                  "prune_pack_batched: tensor %d: group_len %lld is not a multiple of 64 up to 4096 (use surgeon_prune_pack)", i,
                  (long long)p.g);
    if (!A[i] || !mask[i] || (p.k_total > 0 && !vals[i])) return fail(SURGEON_EINVAL, "prune_pack_batched: tensor %d: null pointer", i);
    if (((uintptr_t)A[i] % es) || ((uintptr_t)vals[i] % es) || ((uintptr_t)mask[i] % 8))
      return fail(SURGEON_EINVAL, "prune_pack_batched: tensor %d: misaligned pointer", i);
    if (ceil_div(p.n_groups, 4) > 0x3fffffff) return fail(SURGEON_EUNSUPPORTED, "prune_pack_batched: tensor %d too large", i);
  }
  hipStream_t st = (hipStream_t)stream;
  const int built[10] = {1, 2, 4, 8, 12, 16, 24, 32, 48, 64};
  for (int bi = 0; bi < 10; ++bi) {
    PackBatch bt;
    int count = 0;
    int64_t blocks = 0;
    auto flush = [&]() -> int {
      if (count == 0) return SURGEON_OK;
      for (int j = count; j <= kPackBatch; ++j) bt.first_block[j] = (int)blocks;
      for (int j = count; j < kPackBatch; ++j) {
        bt.A[j] = nullptr; bt.vals[j] = nullptr; bt.mask[j] = nullptr; bt.n_groups[j] = 0;
        bt.g[j] = 64; bt.len_last[j] = 0; bt.k_full[j] = 0; bt.k_last[j] = 0;
      }
      const int rc = dt == SURGEON_F32 ? run_wave_reg_batched<uint32_t>(built[bi], bt, (int)blocks, st)
                                       : run_wave_reg_batched<uint16_t>(built[bi], bt, (int)blocks, st);
      count = 0;
      blocks = 0;
      return rc;
    };
    for (int i = 0; i < l; ++i) {
      const GroupPlan& p = plans[(size_t)i];
      if (p.n == 0 || wave_reg_slots(p.g) != built[bi]) continue;
      if (p.k_total == 0) {  // nothing kept: an all-zero mask, as the single-tensor call writes
        ProfScope prof(SURGEON_PROF_SELECT_OTHER, st);
        const int rc = zero_mask(mask[i], ceil_div(p.n, 64), st);
        if (rc != SURGEON_OK) return rc;
        continue;
      }
      const int64_t b = ceil_div(p.n_groups, 4);
      if (count == kPackBatch || blocks + b > 0x7fffffff) {
        const int rc = flush();
        if (rc != SURGEON_OK) return rc;
      }
      bt.A[count] = A[i]; bt.vals[count] = vals[i]; bt.mask[count] = mask[i]; bt.n_groups[count] = p.n_groups;
      bt.first_block[count] = (int)blocks;
      bt.g[count] = (int)p.g; bt.len_last[count] = (int)p.len_last; bt.k_full[count] = (int)p.k_full; bt.k_last[count] = (int)p.k_last;
      blocks += b;
      ++count;
    }
    const int rc = flush();
    if (rc != SURGEON_OK) return rc;
  }
  return SURGEON_OK;
}
