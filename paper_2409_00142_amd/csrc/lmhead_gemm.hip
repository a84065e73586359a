// LM-head projection for more than 16 hidden rows (batched rounds): an MFMA GEMM.
//
//   logits[r, v] = sum_h hid[r, h] * W[v, h]        (bf16 in, fp32 accumulate, fp32 out)
//
// With hundreds of rows the projection is bound by the matrix cores, not by HBM, and on this chip
// by what feeds them: a 64 x 64 wave tile needs one 1 KB fragment read per MFMA, which measured
// LDS-bound at about a quarter of the MFMA peak.  The kernel therefore uses large wave tiles -
// AB x BB blocks of v_mfma_f32_32x32x16_bf16 per wave, 2 x 2 waves per workgroup, 128 (vocabulary
// rows) x 320 (hidden rows) per workgroup for hundreds of rows - which leaves no registers for
// per-row top-k lists; the fp32 logits of the active rows are written out (HBM has slack in this
// regime) and a second kernel reduces each row (row_topk_kernel).
//
// W is the A operand, so an accumulator lane owns one hidden row and four consecutive vocabulary
// rows per register quad: the output is stored as float4 along V.  Both operands reach LDS by
// LDS-direct loads (16 bytes per lane straight from global memory into LDS: no staging registers,
// no LDS write instructions, nothing returned through the VGPR write path the fragment reads
// use), in tiles of 64 k (one whole 128-byte line per row) that sit in two rings - W tiles four deep,
// hidden-row tiles two to three deep - with one barrier per tile.  Rows are not padded; the eight
// 16-byte chunks of a row are XOR-swizzled with bits 1-3 of the row, which keeps both the
// 1 KB-per-wave copy destinations contiguous and the fragment reads conflict-free.  Only active
// rows are multiplied: the B rows are gathered through the compacted row list and column blocks
// past the last active row are skipped per wave.  Work units are (row tile of W, column tile),
// handed out so that the column tiles of one row tile run on the same XCD and share the W rows
// through its L2.
#include "ddd_device.hpp"
#include "ddd_kernels.hpp"

namespace ddd {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

constexpr int kGK = 64;        // k per LDS tile: 128 bytes per row = one cache line, eight 16-byte chunks
constexpr int kRowB = 2 * kGK; // bytes of a tile row in LDS
constexpr int kWM = 2;         // waves along the vocabulary rows; 2 more along the hidden rows

__device__ __forceinline__ uint32_t bf16_rne(float x) {   // finite inputs; the bf16 bits in the low half
  uint32_t u = __float_as_uint(x);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return u >> 16;
}

// AB x BB blocks of 32 x 32 per wave, 2 x 2 waves per workgroup.  The W tiles (from HBM: long
// latency) and the hidden-row tiles (shared by every workgroup: L2 hits) sit in rings of their own
// depth, as deep as the 160 KB of LDS allow.
template <int AB, int BB>
struct GemmCfg {
  static constexpr int BM = 32 * AB * kWM, BN = 64 * BB;
  static constexpr int kSA = (AB >= 4) ? 3 : 4, kSB = (BB >= 4) ? 2 : 3;   // ring depths, kSB <= kSA
  static constexpr int kABytes = BM * kRowB, kBBytes = BN * kRowB;
  static constexpr int kLdsBytes = kSA * kABytes + kSB * kBBytes;
  static constexpr int NAP = BM / 32, NBP = BN / 32;   // copy instructions per wave and tile (8 rows each)
  static_assert(kSB <= kSA && kLdsBytes <= 160 * 1024, "ring depths");
};

// One work unit of one wave.  The column tile starts at active row tile_col0; this wave multiplies
// NB blocks of 32 rows from block wblk0 of the tile on (0 <= NB <= BB; a wave with NB == 0 still
// copies tiles and meets the barriers).  Every value of NB has its own fully unrolled loop, so the
// accumulators stay in place (no data-dependent branches around the MFMAs).
template <int AB, int BB, int NB>
__device__ __forceinline__ void gemm_unit(const GemmArgs& a, unsigned char* ldsb, int mt, int tile_col0, int wblk0,
                                          int n_act, int tid, int wm, int l32, int lh) {
  using C = GemmCfg<AB, BB>;
  constexpr int NBR = NB > 0 ? NB : 1;
  constexpr int NAP = C::NAP, NBP = C::NBP, kSA = C::kSA, kSB = C::kSB;
  const int KT = a.H / kGK;
  const int col0 = tile_col0 + wblk0 * 32;

  f32x16 acc[AB][NBR];
#pragma unroll
  for (int bm = 0; bm < AB; ++bm)
#pragma unroll
    for (int bn = 0; bn < NBR; ++bn)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[bm][bn][e] = 0.f;

  // ---- copy side: a wave instruction fills 1 KB of LDS = 8 rows x 128 B, each row one whole cache
  // line of its matrix (half lines cost the L1 -> L2 path two requests per line: nothing of a
  // line survives in L1 until the next tile); lane -> (row, 16-byte slot) ----------------------
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  // slot s of tile row r holds chunk s ^ ((r >> 1) & 7); r = (i*4 + wave)*8 + prow
  const int prow = lane >> 3, pc = (lane & 7) ^ ((wave & 1) * 4 + (prow >> 1));
  // byte offsets from the two base pointers (V*H and rows*H elements stay below 2^31).  W is read
  // row-major (a k tile of a row tile = BM pieces of 128 bytes, one per row) or from its tile-major
  // copy (the same pieces contiguous: 256 rows x 128 bytes per block, the next k tile 32 KB on)
  const bool packed = a.Wp != nullptr;
  const unsigned char* Wb = reinterpret_cast<const unsigned char*>(packed ? a.Wp : a.W);
  const uint32_t a_tile_stride = packed ? 256u * kRowB : (uint32_t)kRowB;
  uint32_t ao[NAP], bo[NBP];
#pragma unroll
  for (int i = 0; i < NAP; ++i) {
    const int vrow = mt * C::BM + (i * 4 + wave) * 8 + prow;
    ao[i] = packed ? ((uint32_t)(vrow >> 8) * (uint32_t)KT * 256u + (uint32_t)(vrow & 255)) * kRowB + pc * 16
                   : ((uint32_t)min(vrow, a.V - 1) * (uint32_t)a.H + pc * 8) * 2u;
  }
#pragma unroll
  for (int i = 0; i < NBP; ++i)
    bo[i] = ((uint32_t)a.row_list[min(tile_col0 + (i * 4 + wave) * 8 + prow, n_act - 1)] * (uint32_t)a.H + pc * 8) * 2u;
  typedef const __attribute__((address_space(1))) void* gptr_t;
  typedef __attribute__((address_space(3))) void* lptr_t;
  const unsigned char* Hb = reinterpret_cast<const unsigned char*>(a.hid);
  unsigned char* const ldsA = ldsb;
  unsigned char* const ldsB = ldsb + kSA * C::kABytes;
  // copy instruction i of a tile of W (A) / of the hidden rows (B)
#define DDD_COPY_A(T, STG, i)                                                                        \
  __builtin_amdgcn_global_load_lds((gptr_t)(Wb + (size_t)(T) * a_tile_stride + ao[i]),                       \
                                   (lptr_t)(ldsA + (STG) * C::kABytes + ((i) * 4 + wave) * 1024), 16, 0, 0)
#define DDD_COPY_B(T, STG, i)                                                                        \
  __builtin_amdgcn_global_load_lds((gptr_t)(Hb + (size_t)(T) * kRowB + bo[i]),                       \
                                   (lptr_t)(ldsB + (STG) * C::kBBytes + ((i) * 4 + wave) * 1024), 16, 0, 0)
  // ---- fragment side: lane (l32, lh) of block b reads row b*32 + l32, chunk ks*2 + lh ------------
  const int swz = (l32 >> 1) & 7;   // every tile / block base is a multiple of 32 rows
  int offk[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) offk[ks] = ((ks * 2 + lh) ^ swz) * 16;
  const int arow = (wm * 32 * AB + l32) * kRowB, brow = (wblk0 * 32 + l32) * kRowB;
#define DDD_VMCNT(N) (((N) & 15) | (((N) >> 4) << 14) | (7 << 4) | (15 << 8))
#define DDD_READ(AF, BF, SA, SB, OK)                                                                          \
  {                                                                                                           \
    _Pragma("unroll") for (int b = 0; b < AB; ++b) AF[b] =                                                    \
        __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>((SA) + arow + b * 32 * kRowB + (OK)));     \
    _Pragma("unroll") for (int b = 0; b < NBR; ++b) BF[b] =                                                   \
        __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4*>((SB) + brow + b * 32 * kRowB + (OK)));     \
  }
  // One step = 16 k: the fragments of the next step are read (into the other of two register
  // sets) in front of the MFMAs of this one, so the LDS latency runs under the matrix cores (with
  // one wave per SIMD nothing else would hide it).  The wait for a set is written out, at the end
  // of the MFMA group its reads ran under: left to the compiler it lands behind the reads of the
  // other set and, after an LDS-direct load, always waits for every read in flight.
  // The copy instructions I0 <= i < I1 of the step are spread between its MFMAs: issued in one
  // burst they fill the queue of the address unit, and a wave that cannot issue its next load
  // cannot issue its next MFMA either.
  constexpr int kLgkm0 = (7 << 4) | (0 << 8);     // lgkmcnt(0), expcnt free; the vmcnt bits are added
  constexpr int NM = AB * NBR;                    // MFMAs of a step
#define DDD_WAIT(VM) __builtin_amdgcn_s_waitcnt(kLgkm0 | ((VM) & 15) | (((VM) >> 4) << 14))
#define DDD_STEP(AFN, BFN, SA, SB, OK, AFC, BFC, COPY, T, STG, I0, I1)                                         \
  if (NB > 0) {                                                                                                \
    DDD_READ(AFN, BFN, SA, SB, OK);                                                                            \
    __builtin_amdgcn_sched_barrier(0);                                                                         \
    _Pragma("unroll") for (int mi = 0; mi < NM; ++mi) {                                                        \
      acc[mi % AB][mi / AB] =                                                                                  \
          __builtin_amdgcn_mfma_f32_32x32x16_bf16(AFC[mi % AB], BFC[mi / AB], acc[mi % AB][mi / AB], 0, 0, 0); \
      _Pragma("unroll") for (int ci = (I0); ci < (I1); ++ci) if (((ci - (I0)) * NM) / ((I1) - (I0)) == mi) {   \
        __builtin_amdgcn_sched_barrier(0);                                                                     \
        COPY(T, STG, ci);                                                                                      \
        __builtin_amdgcn_sched_barrier(0);                                                                     \
      }                                                                                                        \
    }                                                                                                          \
    __builtin_amdgcn_sched_barrier(0);                                                                         \
  } else {                                                                                                     \
    _Pragma("unroll") for (int ci = (I0); ci < (I1); ++ci) COPY(T, STG, ci);                                   \
  }
  // Copy schedule.  The barrier of tile kt (in front of its last step) frees the ring slots of
  // tile kt; the hidden rows of tile kt+kSB go there during that last step and the first step of
  // tile kt+1, the W rows of tile kt+kSA during the two middle steps of tile kt+1.  Behind the
  // copies of tile kt+1, which the wait of tile kt needs, each thread then has issued kInFlight more.
  constexpr int NBa = NBP / 2, NAa = NAP / 2;
  constexpr int kInFlight = (kSA - 2) * (NAP + NBP) < NAP + (kSB - 2) * (NAP + NBP) ? (kSA - 2) * (NAP + NBP)
                                                                                      : NAP + (kSB - 2) * (NAP + NBP);
  static_assert(kInFlight < 64, "vmcnt is a 6-bit counter");
  bf16x8 af0[AB], bf0[NBR], af1[AB], bf1[NBR];
  __syncthreads();            // every wave is done with the LDS tiles of the previous unit
  // everything the steps before tile 0 would have issued
#pragma unroll
  for (int p = 0; p < kSA - 1; ++p) {
    if (p < kSB - 1) {
#pragma unroll
      for (int i = 0; i < NBP; ++i) DDD_COPY_B(min(p, KT - 1), p, i);
    }
#pragma unroll
    for (int i = 0; i < NAP; ++i) DDD_COPY_A(min(p, KT - 1), p, i);
  }
#pragma unroll
  for (int i = 0; i < NBa; ++i) DDD_COPY_B(min(kSB - 1, KT - 1), kSB - 1, i);
  __builtin_amdgcn_s_waitcnt(DDD_VMCNT(0));       // all of it has landed: the static count below holds from tile 0 on
  __builtin_amdgcn_s_barrier();
  if (NB > 0) DDD_READ(af0, bf0, ldsA, ldsB, offk[0]);
  DDD_WAIT(63);
  int sa = 0, sb = 0;                             // ring slots of tile kt
  int sap = kSA - 1, sbp = kSB - 1;               // ... and of tile kt-1
  for (int kt = 0; kt < KT; ++kt) {
    const unsigned char* pa = ldsA + sa * C::kABytes;
    const unsigned char* pb = ldsB + sb * C::kBBytes;
    const int sa1 = (sa == kSA - 1) ? 0 : sa + 1, sb1 = (sb == kSB - 1) ? 0 : sb + 1;
    const int tb = min(kt + kSB - 1, KT - 1), ta = min(kt + kSA - 1, KT - 1);   // past the end: the last tile again
    DDD_STEP(af1, bf1, pa, pb, offk[1], af0, bf0, DDD_COPY_B, tb, sbp, NBa, NBP);
    DDD_WAIT(63);
    DDD_STEP(af0, bf0, pa, pb, offk[2], af1, bf1, DDD_COPY_A, ta, sap, 0, NAa);
    DDD_WAIT(63);
    DDD_STEP(af1, bf1, pa, pb, offk[3], af0, bf0, DDD_COPY_A, ta, sap, NAa, NAP);
    // every read of tile kt is back; this thread's copies of tile kt+1 have landed ...
    DDD_WAIT(kInFlight);
    // ... and everybody's; everybody is done with the slots of tile kt, which the next copies overwrite
    // (a plain barrier: __syncthreads() would wait for every load in flight)
    __builtin_amdgcn_s_barrier();
    DDD_STEP(af0, bf0, ldsA + sa1 * C::kABytes, ldsB + sb1 * C::kBBytes, offk[0], af1, bf1, DDD_COPY_B,
             min(kt + kSB, KT - 1), sb, 0, NBa);
    DDD_WAIT(63);
    sap = sa;
    sbp = sb;
    sa = sa1;
    sb = sb1;
  }
  __builtin_amdgcn_s_waitcnt(DDD_VMCNT(0));   // the copies past the end have landed before the LDS is reused
#undef DDD_STEP
#undef DDD_WAIT
#undef DDD_READ
#undef DDD_VMCNT
#undef DDD_COPY_A
#undef DDD_COPY_B

  if (NB == 0) return;
  // accumulator register q*4+e of block (bm, bn): vocabulary row vb + bm*32 + q*8 + e, hidden row column l32
  const int vb = mt * C::BM + wm * 32 * AB + lh * 4;
  const bool v_aligned = (a.V & 3) == 0;
  static_assert(AB % 2 == 0, "a wave covers whole groups of 64 vocabulary rows");
  constexpr int NGW = AB / 2;                                  // groups per wave
  const int grp0 = (mt * C::BM + wm * 32 * AB) >> 6;
  if (a.epi != kGemmLogits) {
    // ---- a linear of the draft layer: store, accumulate, or gate (V is a multiple of 4 there) ------------
#pragma unroll
    for (int bn = 0; bn < NBR; ++bn) {
      const int n = col0 + bn * 32 + l32;
      if (n >= n_act) continue;
      const int orow_id = a.row_list[n];
      float* orow = a.logits + (size_t)orow_id * a.V;
      uint16_t* o16 = a.out16 ? a.out16 + (size_t)orow_id * a.ld16 : nullptr;
      uint16_t* o16b = a.out16b ? a.out16b + (size_t)orow_id * a.ld16 : nullptr;
#pragma unroll
      for (int bm = 0; bm < AB; ++bm)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int v = vb + bm * 32 + q * 8;
          if (v + 3 >= a.V) continue;
          f32x4 o = {acc[bm][bn][q * 4], acc[bm][bn][q * 4 + 1], acc[bm][bn][q * 4 + 2], acc[bm][bn][q * 4 + 3]};
          if (a.epi == kGemmSiluPairs) {   // (v, v+1) and (v+2, v+3) are (gate, up) pairs
            const uint32_t lo = bf16_rne(o[0] / (1.0f + __expf(-o[0])) * o[1]);
            const uint32_t hi = bf16_rne(o[2] / (1.0f + __expf(-o[2])) * o[3]);
            *reinterpret_cast<uint32_t*>(o16 + (v >> 1)) = lo | (hi << 16);
          } else {
            if (a.epi == kGemmAccumulate) o += *reinterpret_cast<const f32x4*>(orow + v);
            *reinterpret_cast<f32x4*>(orow + v) = o;
            if (o16 != nullptr) {
              const uint32_t p0 = bf16_rne(o[0]) | (bf16_rne(o[1]) << 16), p1 = bf16_rne(o[2]) | (bf16_rne(o[3]) << 16);
              *reinterpret_cast<uint2*>(o16 + v) = make_uint2(p0, p1);
              if (o16b != nullptr) *reinterpret_cast<uint2*>(o16b + v) = make_uint2(p0, p1);
            }
          }
        }
    }
    return;
  }
#pragma unroll
  for (int bn = 0; bn < NBR; ++bn) {
    const int n = col0 + bn * 32 + l32;
    // statistics of this hidden row over each group of 64 vocabulary rows the wave covers: each of the two
    // lanes that share the column reduces its 32 values, then the pair is combined (lanes l and l+32)
    float gm[NGW], gs[NGW];
#pragma unroll
    for (int gp = 0; gp < NGW; ++gp) {
      gm[gp] = -INFINITY;
#pragma unroll
      for (int bm = 2 * gp; bm < 2 * gp + 2; ++bm)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int v = vb + bm * 32 + (e >> 2) * 8 + (e & 3);
          const float x = acc[bm][bn][e] + 0.0f;   // -0 -> +0
          acc[bm][bn][e] = x;
          if (v < a.V) gm[gp] = fmaxf(gm[gp], x);
        }
      gm[gp] = fmaxf(gm[gp], __shfl_xor(gm[gp], 32, 64));
      gs[gp] = 0.f;
#pragma unroll
      for (int bm = 2 * gp; bm < 2 * gp + 2; ++bm)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int v = vb + bm * 32 + (e >> 2) * 8 + (e & 3);
          if (v < a.V) gs[gp] += __expf(acc[bm][bn][e] - gm[gp]);
        }
      gs[gp] += __shfl_xor(gs[gp], 32, 64);
    }
    if (n < n_act) {
      const int orow_id = a.row_list[n];
      if (lh == 0) {
#pragma unroll
        for (int gp = 0; gp < NGW; ++gp)
          if ((grp0 + gp) * 64 < a.V) {   // groups past the vocabulary (ragged last tile) are not stored
            a.grp_max[(size_t)orow_id * a.ngrp + grp0 + gp] = gm[gp];
            a.grp_sum[(size_t)orow_id * a.ngrp + grp0 + gp] = gs[gp];
          }
      }
      float* orow = a.logits + (size_t)orow_id * a.V;
#pragma unroll
      for (int bm = 0; bm < AB; ++bm)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int v = vb + bm * 32 + q * 8;
          if (v_aligned && v + 3 < a.V) {
            const f32x4 o = {acc[bm][bn][q * 4], acc[bm][bn][q * 4 + 1], acc[bm][bn][q * 4 + 2],
                             acc[bm][bn][q * 4 + 3]};
            *reinterpret_cast<f32x4*>(orow + v) = o;
          } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
              if (v + e < a.V) orow[v + e] = acc[bm][bn][q * 4 + e];
          }
        }
    }
  }
}

// All work units of one workgroup for column tiles of at most 64 * BB rows.  The blocks of 32
// active rows are dealt evenly: to the column tiles, and inside a tile to the two waves along the
// hidden rows, so that 400 active rows cost 7 + 6 blocks in two tiles of (4, 3) and (3, 3) per
// wave pair instead of 10 + 3 in tiles of (5, 5) and (3, 0).
template <int AB, int BB>
__device__ __forceinline__ void gemm_units(const GemmArgs& a, unsigned char* lds, int n_act, int NT, int bpt) {
  using C = GemmCfg<AB, BB>;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int wm = wave % kWM, wn = wave / kWM;
  const int l32 = lane & 31, lh = lane >> 5;
  const int nmt = (a.V + C::BM - 1) / C::BM;
  const int nblk_all = (n_act + 31) >> 5;
  const int nunits = nmt * NT;
  const int G = gridDim.x;
  const int vg = (blockIdx.x & 7) * (G >> 3) + (blockIdx.x >> 3);   // neighbours on one XCD get neighbouring units

  for (int u = vg; u < nunits; u += G) {
    const int mu = u / NT, nt = u - mu * NT;
    const int mt = a.reverse ? nmt - 1 - mu : mu;   // consecutive calls walk W in opposite directions (memory-side cache)
    const int nblk = min(bpt, nblk_all - nt * bpt);  // >= 1
    const int h0 = (nblk + 1) >> 1;
    const int wblk0 = wn ? h0 : 0, nb = wn ? nblk - h0 : h0;   // wave-uniform
    const int tc0 = nt * bpt * 32;
    switch (nb) {
      case 0: gemm_unit<AB, BB, 0>(a, lds, mt, tc0, wblk0, n_act, tid, wm, l32, lh); break;
      case 1: gemm_unit<AB, BB, 1>(a, lds, mt, tc0, wblk0, n_act, tid, wm, l32, lh); break;
      case 2: gemm_unit<AB, BB, (BB >= 2 ? 2 : BB)>(a, lds, mt, tc0, wblk0, n_act, tid, wm, l32, lh); break;
      case 3: gemm_unit<AB, BB, (BB >= 3 ? 3 : BB)>(a, lds, mt, tc0, wblk0, n_act, tid, wm, l32, lh); break;
      case 4: gemm_unit<AB, BB, (BB >= 4 ? 4 : BB)>(a, lds, mt, tc0, wblk0, n_act, tid, wm, l32, lh); break;
      default: gemm_unit<AB, BB, BB>(a, lds, mt, tc0, wblk0, n_act, tid, wm, l32, lh); break;
    }
  }
}

// BB is the widest column tile the launch may need (64 * BB rows per workgroup).  The number of
// active rows is only known on the device, so the kernel picks the column tiling itself: as few
// tiles as BB allows, the blocks dealt evenly to them, and the narrowest tile that holds a share
// (with 64 active rows a 320-row tile would still copy 320 repeated rows per K tile through LDS).
template <int AB, int BB>
__global__ __launch_bounds__(256, 1) void lmhead_gemm_kernel(GemmArgs a) {
  extern __shared__ __align__(16) unsigned char lds[];     // the two tile rings of the chosen width

  const int n_act = *a.n_act_ptr;
  if (n_act <= 0) return;                                  // uniform
  const int nblk_all = (n_act + 31) >> 5;
  const int NT = (nblk_all + 2 * BB - 1) / (2 * BB);
  const int bpt = (nblk_all + NT - 1) / NT;                // blocks per column tile, <= 2 * BB
  const int bb = (bpt + 1) >> 1;                           // blocks per wave, <= BB
  if (BB >= 5 && bb >= 5)
    gemm_units<AB, (BB >= 5 ? 5 : BB)>(a, lds, n_act, NT, bpt);
  else if (BB >= 4 && bb == 4)
    gemm_units<AB, (BB >= 4 ? 4 : BB)>(a, lds, n_act, NT, bpt);
  else if (BB >= 3 && bb == 3)
    gemm_units<AB, (BB >= 3 ? 3 : BB)>(a, lds, n_act, NT, bpt);
  else if (BB >= 2 && bb == 2)
    gemm_units<AB, (BB >= 2 ? 2 : BB)>(a, lds, n_act, NT, bpt);
  else
    gemm_units<AB, 1>(a, lds, n_act, NT, bpt);
}

// ---- tile-major copy of W ------------------------------------------------------------------------
// One workgroup per (block of 256 rows, block of 64 k); thread t copies the 128 bytes of row t.
__global__ __launch_bounds__(256) void pack_weights_kernel(const uint16_t* __restrict__ W, uint16_t* __restrict__ Wp,
                                                           int V, int H) {
  const int KT = H / kGK;
  const int kt = blockIdx.x % KT, mb = blockIdx.x / KT;
  const int row = min(mb * 256 + (int)threadIdx.x, V - 1);
  const u32x4* src = reinterpret_cast<const u32x4*>(W + (size_t)row * H + (size_t)kt * kGK);
  u32x4* dst = reinterpret_cast<u32x4*>(Wp + ((size_t)blockIdx.x * 256 + threadIdx.x) * kGK);
#pragma unroll
  for (int c = 0; c < 8; ++c) dst[c] = src[c];
}

hipError_t launch_pack_weights(const uint16_t* W, uint16_t* Wp, int V, int H, hipStream_t stream) {
  const int nblk = ((V + 255) / 256) * (H / kGK);
  hipLaunchKernelGGL(pack_weights_kernel, dim3(nblk), dim3(256), 0, stream, W, Wp, V, H);
  return hipGetLastError();
}

// ---- compaction of the active rows ------------------------------------------------------------
__global__ __launch_bounds__(1024) void build_row_list_kernel(const uint8_t* row_active, int n_rows, int32_t* row_list,
                                                              int32_t* n_act) {
  __shared__ int wave_cnt[16];
  __shared__ int base;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (tid == 0) base = 0;
  __syncthreads();
  for (int r0 = 0; r0 < n_rows; r0 += 1024) {
    const int r = r0 + tid;
    const bool on = (r < n_rows) && (row_active == nullptr || row_active[r] != 0);
    const unsigned long long m = __ballot(on);
    if (lane == 0) wave_cnt[wave] = __popcll(m);
    __syncthreads();
    int off = base;
    for (int w = 0; w < wave; ++w) off += wave_cnt[w];
    if (on) row_list[off + __popcll(m & ((1ull << lane) - 1ull))] = r;
    __syncthreads();
    if (tid == 0) {
      int t = 0;
      for (int w = 0; w < 16; ++w) t += wave_cnt[w];
      base += t;
    }
    __syncthreads();
  }
  if (tid == 0) *n_act = base;
}

hipError_t launch_build_row_list(const uint8_t* row_active, int n_rows, int32_t* row_list, int32_t* n_act,
                                 hipStream_t stream) {
  hipLaunchKernelGGL(build_row_list_kernel, dim3(1), dim3(1024), 0, stream, row_active, n_rows, row_list, n_act);
  return hipGetLastError();
}

// Tile shape by the largest number of rows the call can have: 128 x 320 for hundreds of rows,
// smaller column tiles when fewer rows can be active.  (Eight waves on a 256 x 320 tile measured
// a tenth faster with all 640 rows active, but leave half of the CUs idle once fewer than 321
// rows are active, which is most draft calls of a round; four waves on that tile spill.)
// With at most 128 rows and a vocabulary large enough to give every CU a unit, 256 vocabulary rows per
// workgroup (128 x 64 wave tiles) cut the LDS and L2 traffic per MFMA by a quarter.
static int pick_shape(int max_rows, int V, int grid) {
  if (max_rows > 192) return 1;
  if (max_rows > 128) return 2;
  return ((V + 255) / 256 >= grid) ? 4 : 3;
}

template <int AB, int BB>
static hipError_t prepare_shape() {
  return hipFuncSetAttribute(reinterpret_cast<const void*>(&lmhead_gemm_kernel<AB, BB>),
                             hipFuncAttributeMaxDynamicSharedMemorySize, GemmCfg<AB, BB>::kLdsBytes);
}

hipError_t prepare_lmhead_gemm() {
  hipError_t e = prepare_shape<2, 5>();
  if (e == hipSuccess) e = prepare_shape<2, 3>();
  if (e == hipSuccess) e = prepare_shape<2, 2>();
  if (e == hipSuccess) e = prepare_shape<4, 2>();
  return e;
}

template <int AB, int BB>
static void launch_shape(const GemmArgs& a, int grid, hipStream_t stream) {
  constexpr int lds_bytes = GemmCfg<AB, BB>::kLdsBytes;
  hipLaunchKernelGGL((lmhead_gemm_kernel<AB, BB>), dim3(grid), dim3(256), lds_bytes, stream, a);
}

hipError_t launch_gemm_linear(const GemmArgs& a, int max_rows, int grid, hipStream_t stream) {
  // work units of the widest tile that holds the rows; fewer than workgroups: take 128 x 128 tiles instead
  const int mt = (a.V + 127) / 128;
  const int wide = max_rows > 192 ? 320 : max_rows > 128 ? 192 : 128;
  if (mt * ((max_rows + wide - 1) / wide) >= grid) return launch_lmhead_gemm(a, max_rows, grid, stream);
  launch_shape<2, 2>(a, grid, stream);
  return hipGetLastError();
}

hipError_t launch_lmhead_gemm(const GemmArgs& a, int max_rows, int grid, hipStream_t stream) {
  switch (pick_shape(max_rows, a.V, grid)) {
    case 1: launch_shape<2, 5>(a, grid, stream); break;
    case 2: launch_shape<2, 3>(a, grid, stream); break;
    case 4: launch_shape<4, 2>(a, grid, stream); break;
    default: launch_shape<2, 2>(a, grid, stream); break;
  }
  return hipGetLastError();
}

}  // namespace ddd
