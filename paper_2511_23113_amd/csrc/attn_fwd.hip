// Persistent block-sparse flash-attention forward for gfx950 (MI355X), bf16 MFMA, f32 accumulate.
//
// One workgroup per partition walks its own list of work items (head, query block, range of
// the row's active KV blocks).  For every active KV block J of an item it computes, per head,
//   S = scale * Q_I K_J^T,  running row max m and row sum l,  P = exp(S - m),  O += P V_J,
// and ends with O / l and LSE = m + ln l: the block-sparse evaluation of
// O = softmax(Q K^T / sqrt(d)) V (arXiv 2511.23113, Background: "Visual Generative Models",
// "Block-wise Sparse Attention"), where only the dense blocks of the mask are visited, so an
// item costs its number of dense blocks.
//
// Work split inside a workgroup (wave = 64 lanes, lane = 32*g + r):
//   * waves form a (query group) x (key half) grid: wave (a, c) owns QT tiles of 32 query columns
//     and, of every KV block, the keys [c*KW, (c+1)*KW).  Each wave keeps its own running softmax
//     statistics over its key half; the two key halves are combined once per item.
//     Every shape runs QT = 1 (eight waves for 128-token blocks, two for 64-token blocks) at two or
//     three waves per SIMD with everything in the arch-VGPR file: the MFMAs read and write it
//     directly and the softmax reads S in place.  (QT = 2 -- four waves of 64 queries with the
//     accumulators in accumulation registers, one wave per SIMD -- is kept as a template option;
//     it halves the LDS operand reads per MFMA but measured 4-5 % slower.)
//   * Products are formed transposed, S^T = K Q^T and O^T = V^T P^T, with
//     v_mfma_f32_32x32x16_bf16: lane r holds query r, so m and l are per-lane scalars.
//   * S^T's accumulator registers 8h..8h+7 of a 32-key tile hold, in lane group g, the keys
//     16h + {4g..4g+3, 8+4g..8+4g+3}; packed to bf16 they are the B operand of the PV product
//     for that 16-key step.  The matching V^T operand comes from two transposing LDS reads
//     (ds_read_b64_tr_b16) of row-major V: in a group of 16 lanes, lane 4j+a supplies the
//     address of 4 consecutive d-values of key j, and lane i receives d-value i of 4 keys.
// Pair mode (64-token mask blocks, the block size of the paper's PAROAttention masks, at d = 128):
//   the eight-wave workgroup serves two neighbouring query blocks at once, and its KV tile is a pair
//   of 64-token blocks from the union of the two rows' lists; each wave's (query block, KV block)
//   combination carries a flag, and where it is clear the wave's probabilities are exact zeros.
// Software pipeline:
//   the unit of work is 32 keys x (32 QT) queries.  Step i issues, as independent work,
//     the MFMAs of  K Q^T of unit i   and of  V^T P^T of unit i-2,  and
//     the VALU work of the softmax of unit i-1,
//   so matrix and vector pipes run side by side inside one instruction stream (and across the
//   two waves of a SIMD); S and P are double buffered in registers.  A step is a sequence of
//   slots (one V^T P^T MFMA, one K Q^T MFMA, the softmax of two scores per lane, three LDS reads)
//   fenced from each other, and the LDS operands of a slot are read eight MFMAs earlier (those
//   of a step's first half during the step before), so no MFMA waits for a read issued right
//   before it.  The softmax is speculative: probabilities are formed against the running max as
//   it stands; only when a unit's per-lane sum of probabilities exceeds SPEC_SUM_LIMIT (some
//   score is far above the running max) is the unit redone with a raised max and the accumulator
//   rescaled.  The steady state is unrolled over two KV blocks, so LDS buffer offsets are immediates.
// At full occupancy of the chip the kernel runs power-limited (the shader clock drops to about
// 1.8 GHz with all 256 compute units busy, 2.4 GHz with half of them), so instructions and
// bytes saved count as much as cycles saved.
// Data movement:
//   * K and V blocks go L2 -> LDS directly (global_load_lds_dwordx4, 16 bytes per lane, no
//     VGPR staging), double buffered.  There is one barrier per KV block, in the middle of the
//     block's second step; right behind it K of the block after next and V of the next block are
//     copied into the two buffers that barrier retires, so a copy has two steps to land.
//   * LDS tiles are unpadded; 16-byte chunks are XOR-swizzled inside each row instead (the
//     permutation is applied to the per-lane global source address, the LDS side of the copy
//     is linear): K by the row index so that the 16-byte operand reads of 16 lanes (16
//     consecutive keys) hit distinct banks; V by (row & 3) so that the 4 keys of a
//     transposing read hit distinct bank quarters.
#include <hip/hip_runtime.h>

#include <atomic>
#include <cstdint>
#include <type_traits>

#include "fwd_params.hpp"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// The speculative softmax redoes a unit when a lane's sum of its 16 probabilities exceeds this:
// then some score is above the running max by about six powers of two or more (16 probabilities
// at or below 1 sum to less than the limit; until it trips, P may exceed 1 by at most this
// factor, which f32 / bf16 hold without loss).
constexpr float SPEC_SUM_LIMIT = 64.0f;

#define LDS_PTR(T) __attribute__((address_space(3))) T*

__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) {
  f32x2 f = {a, b};
  bf16x2 h = __builtin_convertvector(f, bf16x2);  // round-to-nearest-even
  return __builtin_bit_cast(uint32_t, h);
}

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 u) { return __builtin_bit_cast(bf16x8, u); }

// Exchange between the lane pair (r, r + 32) with one VALU swap of the two 32-lane halves (no
// LDS traffic): v_permlane32_swap swaps the upper half of its first operand with the lower half
// of its second; fed two copies of x it leaves {lo, lo} in the first and {hi, hi} in the second.
// Inline assembly: the compiler's builtin returns the first register for both results.  The
// s_nop's cover the wait states between a VALU write and the swap's read of the same register,
// and between the swap and its consumers, which the compiler cannot insert inside an asm block.
struct halves { float lo, hi; };
__device__ __forceinline__ halves swap_halves(float x) {
  float a = x, b = x;
  asm("s_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\ts_nop 1" : "+v"(a), "+v"(b));
  return {a, b};
}
__device__ __forceinline__ float max_xor32(float x) {
  const halves sw = swap_halves(x);
  return fmaxf(sw.lo, sw.hi);
}
__device__ __forceinline__ float sum_xor32(float x) {
  const halves sw = swap_halves(x);
  return sw.lo + sw.hi;
}

// Direct global -> LDS copies.  One global_load_lds_dwordx4 moves 64 x 16 bytes: lane i reads
// 16 bytes at base + voff(i) + OFF and they land at LDS byte address M0 + OFF + 16*i; the
// instruction offset applies to both sides, so the copies of one group share a base and an M0.
// Inline assembly keeps the copies outside the compiler's wait-count bookkeeping: the kernel
// waits for them explicitly (s_waitcnt vmcnt(0)) right before the barrier that publishes the
// tile.  No "memory" clobber: LDS reads of the OTHER buffer may be scheduled across a copy.
__device__ __forceinline__ void set_copy_dst(uint32_t lds_dst) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0" ::"s"(lds_dst));
}
template <int OFF>
__device__ __forceinline__ void copy16_to_lds(const unsigned char* base, uint32_t voff) {
  asm volatile("global_load_lds_dwordx4 %0, %1 offset:%2" ::"v"(voff), "s"(base), "n"(OFF));
}
// copy number n (0..3) of a group: byte offset n KiB
__device__ __forceinline__ void copy16_nth(int n, const unsigned char* base, uint32_t voff) {
  if (n == 0) copy16_to_lds<0>(base, voff);
  else if (n == 1) copy16_to_lds<1024>(base, voff);
  else if (n == 2) copy16_to_lds<2048>(base, voff);
  else copy16_to_lds<3072>(base, voff);
}

template <int BLK, int D, int QT_>
struct Cfg {
  static constexpr int NQH = BLK / (32 * QT_);   // query groups, one per wave row
  static constexpr int NKH = BLK / 64;      // 64-key groups of a KV block, one per wave column
  static constexpr int NW = NQH * NKH;      // waves
  static constexpr int NT = NW * 64;        // threads
  static constexpr int KW = BLK / NKH;      // keys per wave per KV block
  static constexpr int U = KW / 32;         // 32-key pipeline units per wave per KV block (always 2)
  static_assert(U == 2, "the pipeline below assumes two units per KV block");
  static constexpr int QT = QT_;            // 32-query tiles per wave
  static constexpr int DT = D / 32;         // 32-wide tiles of the head dim
  static constexpr int KS_QK = D / 16;      // k-steps of K Q^T
  static constexpr int NCH = D / 8;         // 16-byte chunks per row
  static constexpr int RPL = 128 / D;       // rows per 256 bytes (one sweep over the 64 LDS banks)
  static constexpr int ROW_BYTES = D * 2;
  static constexpr int TILE_BYTES = BLK * D * 2;
  static constexpr int LOADS = (BLK * D / 8 / 64) / NW;   // 1-KiB direct-to-LDS copies per wave per tile
  static constexpr int RPC = 64 / NCH;                    // tile rows per copy
  // K's swizzle has period NCH*RPL rows: consecutive copies cycle through KVAR per-lane source offsets
  static constexpr int KVAR = (NCH * RPL) / RPC;
  static_assert((LOADS * RPC) % (NCH * RPL) == 0, "a wave's share of a tile must start on a swizzle period");
  static_assert(RPC % (4 * RPL) == 0, "V's swizzle period must divide the rows of one copy");
  static constexpr int NKB = 2, NVB = 2;
  static constexpr int LDS_BYTES = (NKB + NVB) * TILE_BYTES;
  static constexpr int XCH_BYTES = (NKH == 1) ? 0 : NW * (QT * (DT / 2) * 16 * 64 * 4 + QT * 2 * 64 * 4);  // end-of-item exchange
  static_assert(XCH_BYTES <= LDS_BYTES, "exchange area must fit in the tile buffers");
  static_assert(DT % 2 == 0, "the head dim is split between the two key-half waves at the end of an item");
};

template <int BLK, int D, int QT_, bool PAIR>
__global__ __launch_bounds__(BLK * BLK / (32 * QT_)) __attribute__((amdgpu_waves_per_eu(QT_ == 1 ? 2 : 1)))
void dbsp_fwd_kernel(
    const dbsp_fwd_params p, const int32_t* __restrict__ g_row_ptr, const int32_t* __restrict__ g_kv_idx,
    const int4* __restrict__ g_items, const int32_t* __restrict__ g_item_slot,
    const int32_t* __restrict__ g_part_ptr, const int32_t* __restrict__ g_part_items) {
  // the plan's index arrays are read-only for the whole launch: separate __restrict__ const
  // arguments let the compiler fetch them through the scalar unit
  using C = Cfg<BLK, D, QT_>;
  static_assert(!PAIR || (BLK == 128 && D == 128 && QT_ == 1), "pair mode: two 64-token blocks per 128-row tile at d = 128");
  extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];
  constexpr int K_OFF = 0, V_OFF = C::NKB * C::TILE_BYTES;   // byte offsets inside the dynamic LDS block
  const uint32_t lds_base = (uint32_t)(uintptr_t)(LDS_PTR(unsigned char))lds;

  const int t = threadIdx.x;
  const int w = __builtin_amdgcn_readfirstlane(t >> 6);
  const int l = t & 63, r = l & 31, g = l >> 5;
  const int wa = w / C::NKH, wc = w % C::NKH;   // query half, key half
  const int part = blockIdx.x;
  const float c = p.scale_log2;

  // ---- per-lane constants -------------------------------------------------------------
  // direct-to-LDS copies: wave w owns the LOADS consecutive KiB [(w*LOADS + i) KiB, i < LOADS) of
  // every tile.  The LDS tile is a linear image of the global tile except for the chunk swizzle
  // inside a row, which is applied to the per-lane global source offset.
  uint32_t k_src[C::KVAR], v_src;
  {
    const int row_in = l / C::NCH, pch = l % C::NCH;     // row inside the copy, physical chunk
#pragma unroll
    for (int v = 0; v < C::KVAR; ++v) {
      const int row = v * C::RPC + row_in;                // row modulo the swizzle period
      k_src[v] = row_in * C::ROW_BYTES + ((pch ^ ((row / C::RPL) % C::NCH)) * 16);
    }
    v_src = row_in * C::ROW_BYTES + ((pch ^ (((row_in / C::RPL) % (C::NCH / 4)) << 2)) * 16);
  }
  // K operand reads: key row KW*wc + 32*unit + r, logical chunk 2*ks + g, physical chunk
  // (2*ks + g) ^ sw.  Bits 1..3 of the chunk index are ks ^ (sw >> 1), so the address of
  // k-step ks is k_rd0 ^ (ks << 5).
  uint32_t k_rd0;
  {
    const int row = C::KW * wc + r;
    const int sw = (row / C::RPL) % C::NCH;
    k_rd0 = row * C::ROW_BYTES + ((g ^ sw) << 4);
  }
  // V^T operand reads (transposing): lane 4j+a of a 16-lane group addresses key j, d-quad a
  uint32_t v_rd[C::DT];
  {
    const int hh = (l >> 4) & 1, j = (l & 15) >> 2, a4 = l & 3;
    const int key = C::KW * wc + 4 * g + j;
    const int sw = ((key / C::RPL) % (C::NCH / 4)) << 2;
#pragma unroll
    for (int dt = 0; dt < C::DT; ++dt) {
      // V's region offset is part of the per-lane base (kept opaque), so that buffer, unit and
      // k-step offsets of a read fit the instruction's 16-bit immediate
      v_rd[dt] = lds_base + V_OFF + key * C::ROW_BYTES + ((((4 * dt) ^ sw) + 2 * hh + (a4 >> 1)) << 4) + (a4 & 1) * 8;
      asm volatile("" : "+v"(v_rd[dt]));
    }
  }

  uint64_t busy = 0;
  // Work of this workgroup: its own list (once per batch entry), then items from the queue all
  // workgroups share, taken one by one with an atomic counter -- the greedy rule "each unit to the
  // least-loaded partition" (Methodology, "Head-level Partitioning") applied at run time, where
  // "least loaded" is "first to run out of work".
  __shared__ uint32_t tail_pos;
  const int it_begin = g_part_ptr[part], n_own = g_part_ptr[part + 1] - it_begin;
  const int64_t total_own = (int64_t)p.B * n_own;
  const uint32_t total_tail = (uint32_t)p.B * (uint32_t)p.n_tail;
  for (int64_t step_no = 0;; ++step_no) {
    {
      int it, bb;
      if (step_no < total_own) {
        bb = (int)(step_no / n_own);
        it = g_part_items[it_begin + (int)(step_no % n_own)];
      } else {
        if (total_tail == 0) break;
        if (t == 0) tail_pos = atomicAdd(&p.queue[0], 1u);
        __syncthreads();
        const uint32_t pos = __builtin_amdgcn_readfirstlane(tail_pos);
        __syncthreads();                        // everybody has read it before the next take overwrites it
        if (pos >= total_tail) break;
        bb = (int)(pos / (uint32_t)p.n_tail);
        const int tq = (int)(pos % (uint32_t)p.n_tail);
        it = p.tail_items[tq];
        if (t == 0) atomicAdd(&p.queue[2 + tq], 1u);     // take count, read back by dbsp_plan_tail_takes
      }
      const uint64_t t0 = wall_clock64();
      const int4 item = g_items[it];
      const int h = item.x, I = item.y;
      const int slot = g_item_slot[it];
      // this item's KV blocks (pair mode: two words per super block, see block_of / active_in below)
      const int32_t* __restrict__ kv = g_kv_idx + (PAIR ? 2 : 1) * (g_row_ptr[h * p.nQ + I] + item.z);
      const int n_tiles = item.w - item.z;
      const int NU = n_tiles * C::U;                                                  // pipeline units
      const int64_t bh = (int64_t)bb * p.H + h;
      const unsigned char* kbase = reinterpret_cast<const unsigned char*>(p.k + (PAIR ? bh * p.Nk * D : bh * p.nK * BLK * D));
      const unsigned char* vbase = reinterpret_cast<const unsigned char*>(p.v + (PAIR ? bh * p.Nk * D : bh * p.nK * BLK * D));
      // Pair mode: a 128-row tile is two 64-token mask blocks.  Tile T of the item is the super block
      // (j0, j1) = (kv[2T], kv[2T+1] & 0xffffff) with a flag per (query block, KV block) combination in
      // kv[2T+1] >> 24, bit q + 2k.  Wave (wa, wc) works on query block wa / 2 and KV block wc of every
      // super block.  Where its flag is clear it runs the block's stages like everybody (no branches
      // in the step sequence) and forms its probabilities against a running max of +inf, that is, as
      // exact zeros, so the block adds nothing to its sums and its accumulator.  (Leaving those
      // stages out instead, with wave-uniform branches around every group of MFMAs, LDS reads and
      // softmax work, measured 22 % slower with all flags set and no faster at 57 % of them set.)
      // The K / V rows this wave copies (16 w .. 16 w + 15 of the tile) come from block j0 for the
      // first four waves, from j1 for the others.
      auto block_of = [&](int T) -> int {
        if constexpr (PAIR) return (w < C::NW / 2) ? kv[2 * T] : (kv[2 * T + 1] & 0xffffff);
        else return kv[T];
      };
      const int flag_bit = 24 + (wa >> 1) + 2 * wc;
      [[maybe_unused]] auto active_in = [&](int T) -> bool { return ((kv[2 * T + 1] >> flag_bit) & 1) != 0; };
      // this wave's flags of the blocks before, at, after and two after the K Q^T stage's block;
      // the last is fetched next to the id of the same block (see the barrier step), two blocks
      // ahead, so that no step waits for the scalar load
      [[maybe_unused]] bool a_prev = false, a_cur = true, a_next = true, a_next2 = true;
      if constexpr (PAIR) {
        a_cur = active_in(0);
        a_next = (1 < n_tiles) && active_in(1);
      }

      // byte offset of this wave's share inside a tile, same in global memory and in LDS
      const uint32_t wave_off = w * C::LOADS * 1024;
      // one wave's share of a tile: LOADS copies of 1 KiB, in groups of four that share an M0 and a base
      auto copy_k_tile = [&](int J, int buf) {
        const unsigned char* from = PAIR ? kbase + (int64_t)J * (C::TILE_BYTES / 2) + (wave_off & (C::TILE_BYTES / 2 - 1))
                                         : kbase + (int64_t)J * C::TILE_BYTES + wave_off;
        const uint32_t to = lds_base + K_OFF + buf * C::TILE_BYTES + wave_off;
#pragma unroll
        for (int n = 0; n < C::LOADS; ++n) {
          if (n % 4 == 0) set_copy_dst(to + n * 1024);
          copy16_nth(n % 4, from + (n / 4) * 4096, k_src[n % C::KVAR]);
        }
      };
      auto copy_v_tile = [&](int J, int buf) {
        const unsigned char* from = PAIR ? vbase + (int64_t)J * (C::TILE_BYTES / 2) + (wave_off & (C::TILE_BYTES / 2 - 1))
                                         : vbase + (int64_t)J * C::TILE_BYTES + wave_off;
        const uint32_t to = lds_base + V_OFF + buf * C::TILE_BYTES + wave_off;
#pragma unroll
        for (int n = 0; n < C::LOADS; ++n) {
          if (n % 4 == 0) set_copy_dst(to + n * 1024);
          copy16_nth(n % 4, from + (n / 4) * 4096, v_src);
        }
      };
      // Tile schedule: K and V of block T live in buffer T & 1.  K of blocks 0 and 1 and V of block
      // 0 are copied here; from then on the barrier in the middle of block T's second step is
      // followed by the copies of K of block T+2 and V of block T+1, into the buffers whose last
      // reads that barrier has just retired: every copy has two steps to land.
      copy_k_tile(block_of(0), 0);
      if (n_tiles > 1) copy_k_tile(block_of(1), 1);
      copy_v_tile(block_of(0), 0);

      // Q^T operands of this wave's 64 queries: lane (r, g) holds q[32*qt + r][16ks + 8g .. +7]
      const int q0 = 32 * C::QT * wa;
      bf16x8 qreg[C::QT][C::KS_QK];
#pragma unroll
      for (int qt = 0; qt < C::QT; ++qt) {
        // pair mode: the last pair of a head may lack its second query block; its waves load some
        // valid row instead, work on nothing (all their flags are clear) and store nothing
        const int tq = I * BLK + q0 + 32 * qt + r;
        const uint16_t* qrow = PAIR ? p.q + (bh * p.Nq + (tq < p.Nq ? tq : p.Nq - 1)) * D
                                    : p.q + (bh * p.nQ * BLK + (int64_t)I * BLK + q0 + 32 * qt + r) * D;
#pragma unroll
        for (int ks = 0; ks < C::KS_QK; ++ks)
          qreg[qt][ks] = as_bf16x8(*reinterpret_cast<const u32x4*>(qrow + 16 * ks + 8 * g));
      }
      // Make the compiler wait for the Q loads here, before the loop, rather than at their first use
      // inside it (a wait inside the loop would also wait for the in-flight tile copies: same
      // counter; the copies above were issued first, so this wait covers them too).  With eight
      // waves (two per SIMD, 256 registers each) nothing lives in accumulation registers: every MFMA
      // reads and writes the arch-VGPR file and the softmax reads S in place.
#pragma unroll
      for (int qt = 0; qt < C::QT; ++qt)
#pragma unroll
        for (int ks = 0; ks < C::KS_QK; ++ks) {
          if constexpr (C::QT == 1) asm volatile("" : "+v"(qreg[qt][ks]));
          else asm volatile("" : "+a"(qreg[qt][ks]));
        }

      f32x16 oacc[C::DT][C::QT];
#pragma unroll
      for (int dt = 0; dt < C::DT; ++dt)
#pragma unroll
        for (int qt = 0; qt < C::QT; ++qt)
#pragma unroll
          for (int i = 0; i < 16; ++i) oacc[dt][qt][i] = 0.f;
      float m_run[C::QT], mc_run[C::QT], l_run[C::QT];   // running max, the same times scale*log2(e), running sum
#pragma unroll
      for (int qt = 0; qt < C::QT; ++qt) { m_run[qt] = mc_run[qt] = -INFINITY; l_run[qt] = 0.f; }

      // double-buffered pipeline registers: S[x] = scores of the unit whose K Q^T ran in a step of
      // parity x; Pb[x] = its probabilities, packed to bf16 as the B operands of two 16-key steps
      f32x16 S[2][C::QT];
      bf16x8 Pb[2][2][C::QT];
      // The LDS operands of the first half of a step's MFMAs are read during the second half of the
      // step before, those of the second half during the first half: no MFMA waits for a read
      // issued right before it.
      constexpr int KH = C::KS_QK / 2;
      bf16x8 kaA[KH];          // K rows of the next K Q^T unit, k-steps [0, KH)
      s16x4 vaA[C::DT][2];     // V^T operands of the next V^T P^T unit, first 16-key step

      // LDS reads.  K: rows of `half` of the block in buffer `buf`, k-step ks.  V: 16-key step ks of
      // `half` of the block in buffer `buf`, d-tile dt (two transposing reads)
      auto read_k = [&](int buf, int half, int ks) {
        const unsigned char* sK = lds + K_OFF + buf * C::TILE_BYTES + half * 32 * C::ROW_BYTES;
        return as_bf16x8(*reinterpret_cast<const u32x4*>(sK + (k_rd0 ^ (ks << 5))));
      };
      auto read_v = [&](s16x4 (&dst)[2], int buf, int half, int ks, int dt) {
        // absolute LDS byte address as an integer: per-lane base (LDS base and V_OFF inside) plus an
        // offset that is an immediate whenever the buffer parity is static
        const uint32_t vp = v_rd[dt] + buf * C::TILE_BYTES + half * 32 * C::ROW_BYTES + ks * 16 * C::ROW_BYTES;
        dst[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_PTR(s16x4))(uintptr_t)(vp));
        dst[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_PTR(s16x4))(uintptr_t)(vp + 8 * C::ROW_BYTES));
      };

      // id of the block whose V is copied after the next barrier (the block whose K went last)
      int j_v = block_of((1 < n_tiles) ? 1 : 0);

      // One pipeline step.  PAR = parity of the step = half of the KV block its K Q^T unit covers;
      // QK / SM / PV say which stages are live (all three in the steady state; fewer while the
      // pipeline fills and drains); NQK / NPV say the same of the next step, whose first operands
      // this step reads.  The step is a sequence of slots -- two MFMAs, the softmax of two (or
      // four) scores per lane, three LDS reads -- fenced off from each other, so that the matrix
      // pipe always has work queued while the vector work of both waves of a SIMD issues,
      // whatever the phase between the two waves.
      auto step = [&](int i, auto par_tag, auto qk_tag, auto sm_tag, auto pv_tag, auto buf_tag, auto nqk_tag, auto npv_tag) {
        constexpr int PAR = decltype(par_tag)::value;
        // BUF = parity of the KV block of the K Q^T stage when it is known at compile time (steady
        // state: every LDS address is then a loop-invariant register plus an immediate), else -1
        constexpr int BUF = decltype(buf_tag)::value;
        constexpr bool QK = decltype(qk_tag)::value, SM = decltype(sm_tag)::value, PV = decltype(pv_tag)::value;
        constexpr bool NQK = decltype(nqk_tag)::value, NPV = decltype(npv_tag)::value;
        constexpr int HALF = PAR, NHALF = 1 - PAR;
        constexpr bool BAR = QK && HALF == 1;     // the step holds the barrier of its KV block
        // pair mode: does the softmax stage's unit belong to a block this wave works on?  It is in
        // the K Q^T stage's block for the second step of a block, in the block before for the first.
        const bool ls = !PAIR || (PAR == 1 ? a_cur : a_prev);
        const int Tq = i / C::U;                             // block of the K Q^T stage's unit
        const int Tp = (i - 2) / C::U;                       // block of the V^T P^T stage's unit
        static_assert(C::NKB == 2 && C::NVB == 2, "buffer parities below assume double buffering");
        const int bq = (BUF >= 0) ? BUF : (Tq & 1);          // buffer of block Tq
        const int bp = (BUF >= 0) ? 1 - BUF : (Tp & 1);      // buffer of block Tp = Tq - 1
        // next step: its K Q^T unit is the other half of block Tq, or the first half of block Tq+1;
        // its V^T P^T unit is the other half of block Tp, or the first half of block Tp+1
        const int nbq = (HALF == 0) ? bq : 1 - bq, nbp = (HALF == 0) ? bp : 1 - bp;

        bf16x8 kaB[KH];
        s16x4 vaB[C::DT][2];

        // ---- softmax of unit i-1 (VALU), reading S[1-PAR], writing Pb[1-PAR], in eight chunks of
        // two scores.  Speculative: probabilities are formed against the running max as it stands,
        // which is right unless some score is far above it (see SPEC_SUM_LIMIT).
        bool pend = false;
        float l_spec[C::QT], ls0[C::QT], ls1[C::QT];
        uint32_t pw[C::QT][4];
        float mc_eff[C::QT];     // the running max the probabilities are formed against
#pragma unroll
        for (int qt = 0; qt < C::QT; ++qt) {
          mc_eff[qt] = mc_run[qt];
          if constexpr (PAIR) mc_eff[qt] = ls ? mc_run[qt] : INFINITY;   // not this wave's block: exp2(-inf) = 0
        }
        auto softmax_chunk = [&](int j) {     // j = 0..7: scores 2j and 2j+1 of every tile
          const int hf = j / 4, e2 = j % 4;
#pragma unroll
          for (int qt = 0; qt < C::QT; ++qt) {
            const f32x16& sv = S[1 - PAR][qt];
            const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(sv[8 * hf + 2 * e2], c, -mc_eff[qt]));
            const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(sv[8 * hf + 2 * e2 + 1], c, -mc_eff[qt]));
            if (j == 0) { ls0[qt] = p0; ls1[qt] = p1; }      // no "0 + p" to start the two chains
            else { ls0[qt] += p0; ls1[qt] += p1; }
            pw[qt][e2] = pack_bf16x2(p0, p1);
            if (e2 == 3) {
              const u32x4 pb = {pw[qt][0], pw[qt][1], pw[qt][2], pw[qt][3]};
              Pb[1 - PAR][hf][qt] = as_bf16x8(pb);
            }
            if (j == 7) {
              // The test costs one compare (+inf from a running max of -inf, the first unit of an
              // item, trips it too).  Any lane's excess sends the whole wave to the slow path.
              const float lsum = ls0[qt] + ls1[qt];
              pend = pend || (__builtin_amdgcn_ballot_w64(lsum > SPEC_SUM_LIMIT) != 0);
              l_spec[qt] = l_run[qt] + lsum;
            }
          }
        };
        // slow path: p = exp2(s*c - mc) for the 16 scores of tile qt, packed to bf16 into Pb; returns their sum
        auto probabilities = [&](int qt, float mc) {
          const f32x16& sv = S[1 - PAR][qt];
          float a0 = 0.f, a1 = 0.f;
#pragma unroll
          for (int hf = 0; hf < 2; ++hf) {
            uint32_t w4[4];
#pragma unroll
            for (int e2 = 0; e2 < 4; ++e2) {
              const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(sv[8 * hf + 2 * e2], c, -mc));
              const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(sv[8 * hf + 2 * e2 + 1], c, -mc));
              a0 += p0;
              a1 += p1;
              w4[e2] = pack_bf16x2(p0, p1);
            }
            const u32x4 pb = {w4[0], w4[1], w4[2], w4[3]};
            Pb[1 - PAR][hf][qt] = as_bf16x8(pb);
          }
          return a0 + a1;
        };
        // slow path: largest of this lane's 16 scores of tile qt, two chains of 3-input maxima
        auto lane_max = [&](int qt) {
          const f32x16& sv = S[1 - PAR][qt];
          float mx0 = fmaxf(fmaxf(sv[0], sv[1]), sv[2]), mx1 = fmaxf(fmaxf(sv[3], sv[4]), sv[5]);
          mx0 = fmaxf(fmaxf(mx0, sv[6]), sv[7]);
          mx1 = fmaxf(fmaxf(mx1, sv[8]), sv[9]);
          mx0 = fmaxf(fmaxf(mx0, sv[10]), sv[11]);
          mx1 = fmaxf(fmaxf(mx1, sv[12]), sv[13]);
          mx0 = fmaxf(fmaxf(mx0, sv[14]), sv[15]);
          return fmaxf(mx0, mx1);
        };

        auto mfma_pv = [&](const s16x4 (&va)[2], int ks, int dt) {
          const bf16x8 a = __builtin_bit_cast(bf16x8, __builtin_shufflevector(va[0], va[1], 0, 1, 2, 3, 4, 5, 6, 7));
#pragma unroll
          for (int qt = 0; qt < C::QT; ++qt)
            oacc[dt][qt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, Pb[PAR][ks][qt], oacc[dt][qt], 0, 0, 0);
        };
        auto mfma_qk = [&](const bf16x8& ka, int ks) {
#pragma unroll
          for (int qt = 0; qt < C::QT; ++qt) {
            if (ks == 0) {
#pragma unroll
              for (int e = 0; e < 16; ++e) S[PAR][qt][e] = 0.f;
            }
            S[PAR][qt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qreg[qt][ks], S[PAR][qt], 0, 0, 0);
          }
        };
        // a half step holds DT d-tiles of V^T P^T and KH k-steps of K Q^T (DT == KH): slot x pairs them
        static_assert(C::DT == KH, "a slot pairs one d-tile of V^T P^T with one k-step of K Q^T");
        constexpr int SLOTS = KH, CPS = 4 / SLOTS;     // softmax chunks per slot
        static_assert(SLOTS * CPS == 4, "four softmax chunks per half step");

        // ---- first half: MFMAs on the operands read during the previous step; reads for the second half
        int jk = 0;
        [[maybe_unused]] int kw0 = 0, kw1 = 0;
#pragma unroll
        for (int x = 0; x < SLOTS; ++x) {
          if constexpr (QK) kaB[x] = read_k(bq, HALF, KH + x);
          if constexpr (PV) read_v(vaB[x], bp, HALF, 1, x);
          if constexpr (PV) mfma_pv(vaA[x], 0, x);
          if constexpr (QK) mfma_qk(kaA[x], x);
          if constexpr (SM) {
#pragma unroll
            for (int cc = 0; cc < CPS; ++cc) softmax_chunk(x * CPS + cc);
          }
          if constexpr (BAR) {
            // id of the block whose K is copied after the barrier below, through the scalar cache
            // (pair mode: the two words of that super block; they are taken apart behind the
            // barrier, whose wait covers the loads, so that nothing here waits for them)
            if (x == SLOTS - 1) {
              const int Tn = (Tq + 2 < n_tiles) ? Tq + 2 : n_tiles - 1;
              if constexpr (PAIR) { kw0 = kv[2 * Tn]; kw1 = kv[2 * Tn + 1]; }
              else jk = kv[Tn];
            }
          }
          __builtin_amdgcn_sched_barrier(0);
        }
        if constexpr (BAR) {
          // One barrier per KV block.  Before it, this wave's copies have landed and its reads of
          // block Tq's K and block Tq-1's V are complete; after it, everybody's: K of block Tq+1 and
          // V of block Tq may be read, and the two retired buffers are refilled.
          if constexpr (SM) {   // the first half of the softmax stays on this side (see the pin further down)
#pragma unroll
            for (int qt = 0; qt < C::QT; ++qt) asm volatile("" ::"v"(Pb[1 - PAR][0][qt]), "v"(ls0[qt]), "v"(ls1[qt]));
          }
          asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
          __syncthreads();
          if constexpr (PAIR) {
            jk = (w < C::NW / 2) ? kw0 : (kw1 & 0xffffff);
            a_next2 = (Tq + 2 < n_tiles) && ((kw1 >> flag_bit) & 1) != 0;
          }
          if (Tq + 2 < n_tiles) copy_k_tile(jk, bq);
          if (Tq + 1 < n_tiles) copy_v_tile(j_v, 1 - bq);
          j_v = jk;
        }
        // ---- second half: MFMAs on the operands read in the first half; reads for the next step
#pragma unroll
        for (int x = 0; x < SLOTS; ++x) {
          if constexpr (NQK) kaA[x] = read_k(nbq, NHALF, x);
          if constexpr (NPV) read_v(vaA[x], nbp, NHALF, 0, x);
          if constexpr (PV) mfma_pv(vaB[x], 1, x);
          if constexpr (QK) mfma_qk(kaB[x], KH + x);
          if constexpr (SM) {
#pragma unroll
            for (int cc = 0; cc < CPS; ++cc) softmax_chunk(4 + x * CPS + cc);
          }
          __builtin_amdgcn_sched_barrier(0);
        }
        if constexpr (PAIR && BAR) { a_prev = a_cur; a_cur = a_next; a_next = a_next2; }   // on to the next block

        // ---- slow path: raise the running max, redo the probabilities, rescale the accumulator
        //      (after V^T P^T of unit i-2, before that of unit i-1) ------------------------------
        if constexpr (SM) {
          // pin the speculative results here: otherwise the compiler sinks the conversions below
          // the (rarely taken) branch, out of the slots whose MFMAs they are meant to overlap with
#pragma unroll
          for (int qt = 0; qt < C::QT; ++qt) {
            asm volatile("" ::"v"(Pb[1 - PAR][0][qt]), "v"(Pb[1 - PAR][1][qt]), "v"(l_spec[qt]));
          }
          if (pend) {
#pragma unroll
            for (int qt = 0; qt < C::QT; ++qt) {
              const float m_new = fmaxf(m_run[qt], max_xor32(lane_max(qt)));
              const float alpha = __builtin_amdgcn_exp2f((m_run[qt] - m_new) * c);
              m_run[qt] = m_new;
              mc_run[qt] = m_new * c;
              l_spec[qt] = l_run[qt] * alpha + probabilities(qt, mc_run[qt]);
#pragma unroll
              for (int dt = 0; dt < C::DT; ++dt)
#pragma unroll
                for (int e = 0; e < 16; ++e) oacc[dt][qt][e] *= alpha;
            }
          }
#pragma unroll
          for (int qt = 0; qt < C::QT; ++qt) l_run[qt] = l_spec[qt];
        }
      };

      using T0 = std::integral_constant<int, 0>;
      using T1 = std::integral_constant<int, 1>;
      using Yes = std::true_type;
      using No = std::false_type;
      using B0 = std::integral_constant<int, 0>;
      using B1 = std::integral_constant<int, 1>;
      using Bx = std::integral_constant<int, -1>;
      // K of block 0 is there for everybody: read the first operands of step 0
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      __syncthreads();
#pragma unroll
      for (int x = 0; x < KH; ++x) kaA[x] = read_k(0, 0, x);
      // fill (two steps), steady state, drain (two steps); NU is even, so parities are static.  A
      // step may read K operands for a K Q^T stage that does not follow (last block): they are
      // stale LDS contents and go unused.
      step(0, T0{}, Yes{}, No{}, No{}, B0{}, Yes{}, No{});
      step(1, T1{}, Yes{}, Yes{}, No{}, B0{}, Yes{}, Yes{});
      int i = 2;
      for (; i + 2 < NU; i += 4) {           // two KV blocks per trip: odd block, then even block
        step(i, T0{}, Yes{}, Yes{}, Yes{}, B1{}, Yes{}, Yes{});
        step(i + 1, T1{}, Yes{}, Yes{}, Yes{}, B1{}, Yes{}, Yes{});
        step(i + 2, T0{}, Yes{}, Yes{}, Yes{}, B0{}, Yes{}, Yes{});
        step(i + 3, T1{}, Yes{}, Yes{}, Yes{}, B0{}, Yes{}, Yes{});
      }
      if (i < NU) {                          // one odd block left
        step(i, T0{}, Yes{}, Yes{}, Yes{}, B1{}, Yes{}, Yes{});
        step(i + 1, T1{}, Yes{}, Yes{}, Yes{}, B1{}, Yes{}, Yes{});
      }
      step(NU, T0{}, No{}, Yes{}, Yes{}, Bx{}, No{}, Yes{});
      step(NU + 1, T1{}, No{}, No{}, Yes{}, Bx{}, No{}, No{});

      // ---- end of item: combine the key halves (if the block has two) and store ----------------
      __syncthreads();   // every wave is done reading the K/V tiles: the buffers become the exchange area
      const int64_t tok0 = PAIR ? bh * p.Nq + (int64_t)I * BLK + q0 + r : bh * p.nQ * BLK + (int64_t)I * BLK + q0 + r;
      // pair mode: false for the waves of a query block past the end of the head (they still fill
      // their rows of a split row's partial result: zeros and -inf)
      const bool q_there = !PAIR || I * BLK + q0 < p.Nq;
      const int64_t ps = (int64_t)bb * p.n_slots + slot;
      // stores 16 values of one 32x32 tile of O^T: query tok, d = 32*dt + 8*(e/4) + 4*g + e%4
      auto store_tile = [&](const float (&res)[16], int64_t tok, int qloc, int dt) {
        if (slot < 0) {
          if (!q_there) return;
          uint16_t* orow = p.o + tok * D + 32 * dt + 4 * g;
#pragma unroll
          for (int i4 = 0; i4 < 4; ++i4) {
            u32x2 pk;
            pk.x = pack_bf16x2(res[4 * i4 + 0], res[4 * i4 + 1]);
            pk.y = pack_bf16x2(res[4 * i4 + 2], res[4 * i4 + 3]);
            *reinterpret_cast<u32x2*>(orow + 8 * i4) = pk;
          }
        } else {
          float* orow = p.part_o + (ps * BLK + qloc) * D + 32 * dt + 4 * g;
#pragma unroll
          for (int i4 = 0; i4 < 4; ++i4) {
            f32x4 f = {res[4 * i4 + 0], res[4 * i4 + 1], res[4 * i4 + 2], res[4 * i4 + 3]};
            *reinterpret_cast<f32x4*>(orow + 8 * i4) = f;
          }
        }
      };
      auto store_lse = [&](float lse, int64_t tok, int qloc) {
        if (slot < 0) { if (p.lse != nullptr && q_there) p.lse[tok] = lse; }
        else p.part_lse[ps * BLK + qloc] = lse;
      };

      if constexpr (C::NKH == 1) {
#pragma unroll
        for (int qt = 0; qt < C::QT; ++qt) {
          const float lt = sum_xor32(l_run[qt]);
          const float inv = 1.0f / lt;
          const int64_t tok = tok0 + 32 * qt;
#pragma unroll
          for (int dt = 0; dt < C::DT; ++dt) {
            float res[16];
#pragma unroll
            for (int e = 0; e < 16; ++e) res[e] = oacc[dt][qt][e] * inv;
            store_tile(res, tok, q0 + 32 * qt + r, dt);
          }
          if (g == 0) store_lse(m_run[qt] * p.scale + __logf(lt), tok, q0 + 32 * qt + r);
        }
      } else {
        // wave (a, c) finalises d-tiles [c*DT/2, (c+1)*DT/2) and hands the other half to its partner
        constexpr int HT = C::DT / 2;
        float* xo = reinterpret_cast<float*>(lds) + w * (C::QT * HT * 16 * 64);
        float* xs = reinterpret_cast<float*>(lds) + C::NW * (C::QT * HT * 16 * 64) + w * (C::QT * 2 * 64);
        const int pw = wa * C::NKH + (1 - wc);   // partner wave: same queries, other key half
        const float* yo = reinterpret_cast<const float*>(lds) + pw * (C::QT * HT * 16 * 64);
        const float* ys = reinterpret_cast<const float*>(lds) + C::NW * (C::QT * HT * 16 * 64) + pw * (C::QT * 2 * 64);
        // WC is this wave's key half as a compile-time constant, so that the accumulator tiles
        // are addressed with constant indices (they must stay in registers)
        auto finish = [&](auto wc_tag) {
          constexpr int WC = decltype(wc_tag)::value;
          float l_full[C::QT];
#pragma unroll
          for (int qt = 0; qt < C::QT; ++qt) {
            l_full[qt] = sum_xor32(l_run[qt]);
            xs[(2 * qt + 0) * 64 + l] = m_run[qt];
            xs[(2 * qt + 1) * 64 + l] = l_full[qt];
#pragma unroll
            for (int hx = 0; hx < HT; ++hx)
#pragma unroll
              for (int e = 0; e < 16; ++e) xo[((qt * HT + hx) * 16 + e) * 64 + l] = oacc[(1 - WC) * HT + hx][qt][e];
          }
          __syncthreads();
#pragma unroll
          for (int qt = 0; qt < C::QT; ++qt) {
            const float mp = ys[(2 * qt + 0) * 64 + l], lp = ys[(2 * qt + 1) * 64 + l];
            const float mt = fmaxf(m_run[qt], mp);
            // pair mode: a query block may have nothing in this item (both halves at -inf, sums 0):
            // its rows come out as O = 0, LSE = -inf, without forming inf - inf or 0 / 0
            const float mref = (PAIR && mt == -INFINITY) ? 0.f : mt;
            const float fs = __builtin_amdgcn_exp2f((m_run[qt] - mref) * c);
            const float fp = __builtin_amdgcn_exp2f((mp - mref) * c);
            const float lt = l_full[qt] * fs + lp * fp;
            const float inv = (PAIR && !(lt > 0.f)) ? 0.f : 1.0f / lt;
            const float fsi = fs * inv, fpi = fp * inv;
            const int64_t tok = tok0 + 32 * qt;
#pragma unroll
            for (int hx = 0; hx < HT; ++hx) {
              float res[16];
#pragma unroll
              for (int e = 0; e < 16; ++e)
                res[e] = oacc[WC * HT + hx][qt][e] * fsi + yo[((qt * HT + hx) * 16 + e) * 64 + l] * fpi;
              store_tile(res, tok, q0 + 32 * qt + r, WC * HT + hx);
            }
            if (WC == 0 && g == 0) store_lse(mt * p.scale + __logf(lt), tok, q0 + 32 * qt + r);
          }
        };
        if (wc == 0) finish(std::integral_constant<int, 0>{});
        else finish(std::integral_constant<int, 1>{});
        __syncthreads();   // exchange area fully read before the next item's copies overwrite it
      }
      busy += wall_clock64() - t0;
    }
  }

  if (t == 0) {
    if (total_tail != 0) {
      // The last workgroup to leave rewinds the queue for the next launch: by then every workgroup
      // has made its last (failing) take.
      __threadfence();
      if (atomicAdd(&p.queue[1], 1u) == gridDim.x - 1) {
        p.queue[0] = 0;
        p.queue[1] = 0;
        __threadfence();
      }
    }
    p.busy[part] = busy;
    const uint32_t hw = __builtin_amdgcn_s_getreg((31 << 11) | (0 << 6) | 4);    // HW_ID
    const uint32_t xcc = __builtin_amdgcn_s_getreg((3 << 11) | (0 << 6) | 20);   // XCC_ID[3:0]
    const uint32_t cu = (hw >> 8) & 0xf, sh = (hw >> 12) & 0x1, se = (hw >> 13) & 0x7;
    p.hw_id[part] = (xcc << 16) | (se << 8) | (sh << 4) | cu;
  }
}

// Fix-up pass: merges the chunks of split rows (log-sum-exp identity, the same one that
// combines per-chunk partial attention in Ring Attention) and fills rows with no active block.
//   LSE = log sum_k exp(LSE_k),  O = sum_k exp(LSE_k - LSE) O_k;   empty row: O = 0, LSE = -inf.
// Grid: (B * (n_split + n_empty), blk * D / 4 / 256) workgroups of 256 threads; a thread produces four
// consecutive d-values of one query (all its loads are independent of each other: the pass is
// bandwidth-bound, not latency-bound).
// blk = query rows of a plan row (pair mode: 128, where the last row of a head may reach past Nq
// by one 64-token block and a query block may have no active block in some or all chunks).
template <int D>
__global__ __launch_bounds__(256) void dbsp_fixup_kernel(const dbsp_fwd_params p, int blk) {
  const int per_b = p.n_split + p.n_empty;
  const int bb = blockIdx.x / per_b, e = blockIdx.x % per_b;
  const int x = blockIdx.y * 256 + threadIdx.x;          // < blk * D / 4
  const int qloc = x / (D / 4), d4 = x % (D / 4);
  if (e < p.n_split) {
    const int4 sr = reinterpret_cast<const int4*>(p.split_rows)[e];
    const int row = sr.x, first = sr.y, nch = sr.z;
    const int h = row / p.nQ, I = row % p.nQ;
    const int64_t bh = (int64_t)bb * p.H + h;
    const int64_t ps0 = (int64_t)bb * p.n_slots + first;
    if (I * blk + qloc >= p.Nq) return;
    float mx = -INFINITY;
    for (int kx = 0; kx < nch; ++kx) mx = fmaxf(mx, p.part_lse[(ps0 + kx) * blk + qloc]);
    const bool none = (mx == -INFINITY);      // no chunk has anything for this query: O = 0, LSE = -inf
    const float mref = none ? 0.f : mx;
    float tot = 0.f;
    for (int kx = 0; kx < nch; ++kx) tot += __expf(p.part_lse[(ps0 + kx) * blk + qloc] - mref);
    const float lse = none ? -INFINITY : mx + __logf(tot);
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    for (int kx = 0; kx < nch; ++kx) {
      const float wgt = none ? 0.f : __expf(p.part_lse[(ps0 + kx) * blk + qloc] - lse);
      const f32x4 f = *reinterpret_cast<const f32x4*>(p.part_o + ((ps0 + kx) * blk + qloc) * D + 4 * d4);
      acc.x += wgt * f.x;  acc.y += wgt * f.y;  acc.z += wgt * f.z;  acc.w += wgt * f.w;
    }
    const int64_t tok = bh * p.Nq + (int64_t)I * blk + qloc;
    u32x2 pk;
    pk.x = pack_bf16x2(acc.x, acc.y);
    pk.y = pack_bf16x2(acc.z, acc.w);
    *reinterpret_cast<u32x2*>(p.o + tok * D + 4 * d4) = pk;
    if (p.lse != nullptr && d4 == 0) p.lse[tok] = lse;
  } else {
    const int row = p.empty_rows[e - p.n_split];
    const int h = row / p.nQ, I = row % p.nQ;
    const int64_t bh = (int64_t)bb * p.H + h;
    if (I * blk + qloc >= p.Nq) return;
    const int64_t tok = bh * p.Nq + (int64_t)I * blk + qloc;
    *reinterpret_cast<u32x2*>(p.o + tok * D + 4 * d4) = u32x2{0u, 0u};
    if (p.lse != nullptr && d4 == 0) p.lse[tok] = -INFINITY;
  }
}

template <int BLK, int D, int QT_, bool PAIR = false>
hipError_t launch_fwd(const dbsp_fwd_params& p, int P, hipStream_t stream) {
  using C = Cfg<BLK, D, QT_>;
  // the dynamic-LDS limit is a per-device function attribute: set it once per device
  static std::atomic<uint32_t> attr_set_mask{0};
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  const uint32_t bit = 1u << (dev & 31);
  if (!(attr_set_mask.load(std::memory_order_acquire) & bit)) {
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(&dbsp_fwd_kernel<BLK, D, QT_, PAIR>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, C::LDS_BYTES);
    if (e != hipSuccess) return e;
    attr_set_mask.fetch_or(bit, std::memory_order_release);
  }
  hipLaunchKernelGGL((dbsp_fwd_kernel<BLK, D, QT_, PAIR>), dim3(P), dim3(C::NT), C::LDS_BYTES, stream, p, p.row_ptr, p.kv_idx,
                     reinterpret_cast<const int4*>(p.items), p.item_slot, p.part_ptr, p.part_items);
  return hipGetLastError();
}

}  // namespace

hipError_t dbsp_launch_fwd(const dbsp_fwd_params& p, int block, int d, bool pair, int P, hipStream_t stream) {
  hipError_t e;
  if (pair && (block != 64 || d != 128)) return hipErrorInvalidValue;
  // waves of 32 queries everywhere: eight per workgroup for 128-token blocks, two for 64-token blocks
  if (pair) { e = launch_fwd<128, 128, 1, true>(p, P, stream); block = 128; }
  else if (block == 128 && d == 128) e = launch_fwd<128, 128, 1>(p, P, stream);
  else if (block == 128 && d == 64) e = launch_fwd<128, 64, 1>(p, P, stream);
  else if (block == 64 && d == 128) e = launch_fwd<64, 128, 1>(p, P, stream);
  else if (block == 64 && d == 64) e = launch_fwd<64, 64, 1>(p, P, stream);
  else return hipErrorInvalidValue;
  if (e != hipSuccess) return e;
  const int fix = p.B * (p.n_split + p.n_empty);
  if (fix > 0) {
    const dim3 grid(fix, block * d / 4 / 256);      // block >= 64 and d >= 64: a whole number of workgroups per row
    if (d == 128) hipLaunchKernelGGL((dbsp_fixup_kernel<128>), grid, dim3(256), 0, stream, p, block);
    else hipLaunchKernelGGL((dbsp_fixup_kernel<64>), grid, dim3(256), 0, stream, p, block);
    e = hipGetLastError();
  }
  return e;
}
