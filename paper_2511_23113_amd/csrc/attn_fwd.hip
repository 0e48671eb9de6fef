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
// Work split inside a workgroup (wave = 64 lanes, lane = 32*g + r, 16-lane group index hh):
//   * waves form a (query half) x (key half) grid: wave (a, c) owns 64 query columns and, of
//     every KV block, the keys [c*KW, (c+1)*KW).  Each wave keeps its own running softmax
//     statistics over its key half; the two key halves are combined once per item.
//   * Products are formed transposed, S^T = K Q^T and O^T = V^T P^T, with
//     v_mfma_f32_32x32x16_bf16: lane r holds query r, so m and l are per-lane scalars, and a
//     K (or V^T) operand read from LDS feeds two MFMAs (the wave's two 32-query tiles).
//   * S^T's accumulator registers 8h..8h+7 of a 32-key tile hold, in lane group g, the keys
//     16h + {4g..4g+3, 8+4g..8+4g+3}; packed to bf16 they are the B operand of the PV product
//     for that 16-key step.  The matching V^T operand comes from two transposing LDS reads
//     (ds_read_b64_tr_b16) of row-major V: in a group of 16 lanes, lane 4j+a supplies the
//     address of 4 consecutive d-values of key j, and lane i receives d-value i of 4 keys.
// Data movement:
//   * K and V blocks go HBM/L2 -> LDS directly (global_load_lds_dwordx4, 16 bytes per lane,
//     no VGPR staging), double buffered: the loads of block j+1 fly while block j is computed.
//   * LDS tiles are unpadded; 16-byte chunks are XOR-swizzled inside each row instead (the
//     permutation is applied to the per-lane global source address, the LDS side of the copy
//     is linear): K by the row index so that the 16-byte operand reads of 16 lanes (16
//     consecutive keys) hit distinct banks; V by (row & 3) so that the 4 keys of a
//     transposing read hit distinct bank quarters.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <type_traits>

#include "fwd_params.hpp"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

#define LDS_PTR(T) __attribute__((address_space(3))) T*
#define GLOBAL_PTR(T) __attribute__((address_space(1))) T*

__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) {
  f32x2 f = {a, b};
  bf16x2 h = __builtin_convertvector(f, bf16x2);  // round-to-nearest-even
  return __builtin_bit_cast(uint32_t, h);
}

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 u) { return __builtin_bit_cast(bf16x8, u); }

__device__ __forceinline__ float xor32(float x) { return __shfl_xor(x, 32, 64); }

template <int BLK, int D>
struct Cfg {
  static constexpr int NQH = BLK / 64;      // 64-query groups
  static constexpr int NKH = 2;             // key halves
  static constexpr int NW = NQH * NKH;      // waves
  static constexpr int NT = NW * 64;        // threads
  static constexpr int KW = BLK / NKH;      // keys per wave per KV block
  static constexpr int KTW = KW / 32;       // 32-key tiles per wave
  static constexpr int QT = 2;              // 32-query tiles per wave
  static constexpr int DT = D / 32;         // 32-wide tiles of the head dim
  static constexpr int KS_QK = D / 16;      // k-steps of K Q^T
  static constexpr int KS_PV = KW / 16;     // k-steps of V^T P^T (per wave)
  static constexpr int NCH = D / 8;         // 16-byte chunks per row
  static constexpr int RPL = 128 / D;       // rows per 256 bytes (one sweep over the 64 LDS banks)
  static constexpr int ROW_BYTES = D * 2;
  static constexpr int TILE_BYTES = BLK * D * 2;
  static constexpr int LOADS = (BLK * D / 8 / 64) / NW;   // 1-KiB direct-to-LDS copies per wave per tile
  static constexpr int LDS_BYTES = 4 * TILE_BYTES;        // K[2], V[2]
  static constexpr int XCH_BYTES = NW * (QT * (DT / 2) * 16 * 64 * 4 + QT * 2 * 64 * 4);  // end-of-item exchange
  static_assert(XCH_BYTES <= LDS_BYTES, "exchange area must fit in the tile buffers");
  static_assert(DT % 2 == 0, "the head dim is split between the two key-half waves at the end of an item");
};

template <int BLK, int D>
__global__ __launch_bounds__(BLK * 2) void dbsp_fwd_kernel(
    const dbsp_fwd_params p, const int32_t* __restrict__ g_row_ptr, const int32_t* __restrict__ g_kv_idx,
    const int4* __restrict__ g_items, const int32_t* __restrict__ g_item_slot,
    const int32_t* __restrict__ g_part_ptr, const int32_t* __restrict__ g_part_items) {
  // the plan's index arrays are read-only for the whole launch: separate __restrict__ const
  // arguments let the compiler fetch them through the scalar unit
  using C = Cfg<BLK, D>;
  extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];
  // byte offsets inside the dynamic LDS block
  constexpr int K_OFF = 0, V_OFF = 2 * C::TILE_BYTES;

  const int t = threadIdx.x;
  const int w = __builtin_amdgcn_readfirstlane(t >> 6);
  const int l = t & 63, r = l & 31, g = l >> 5;
  const int wa = w / C::NKH, wc = w % C::NKH;   // query half, key half
  const int part = blockIdx.x;
  const float c = p.scale_log2;

  // ---- per-lane constants -------------------------------------------------------------
  // direct-to-LDS copies: copy i of this wave fills LDS chunks [(i*NW + w)*64, +64) of a tile
  uint32_t k_src[C::LOADS], v_src[C::LOADS];
#pragma unroll
  for (int i = 0; i < C::LOADS; ++i) {
    const int pc = (i * C::NW + w) * 64 + l;            // physical chunk
    const int row = pc / C::NCH, pch = pc % C::NCH;
    const int kch = pch ^ ((row / C::RPL) % C::NCH);
    const int vch = pch ^ (((row / C::RPL) % (C::NCH / 4)) << 2);
    k_src[i] = row * C::ROW_BYTES + kch * 16;
    v_src[i] = row * C::ROW_BYTES + vch * 16;
  }
  // K operand reads: key row KW*wc + 32*kt + r, logical chunk 2*ks + g
  uint32_t k_rd[C::KS_QK];
  {
    const int row = C::KW * wc + r;
    const int sw = (row / C::RPL) % C::NCH;
#pragma unroll
    for (int ks = 0; ks < C::KS_QK; ++ks) k_rd[ks] = row * C::ROW_BYTES + (((2 * ks + g) ^ sw) << 4);
  }
  // V^T operand reads (transposing): lane 4j+a of a 16-lane group addresses key j, d-quad a
  uint32_t v_rd[C::DT];
  {
    const int hh = (l >> 4) & 1, j = (l & 15) >> 2, a4 = l & 3;
    const int key = C::KW * wc + 4 * g + j;
    const int sw = ((key / C::RPL) % (C::NCH / 4)) << 2;
#pragma unroll
    for (int dt = 0; dt < C::DT; ++dt)
      v_rd[dt] = key * C::ROW_BYTES + ((((4 * dt) ^ sw) + 2 * hh + (a4 >> 1)) << 4) + (a4 & 1) * 8;
  }

  uint64_t busy = 0;
  const int it_begin = g_part_ptr[part], it_end = g_part_ptr[part + 1];
  for (int bb = 0; bb < p.B; ++bb) {
    for (int ii = it_begin; ii < it_end; ++ii) {
      const uint64_t t0 = wall_clock64();
      const int it = g_part_items[ii];
      const int4 item = g_items[it];
      const int h = item.x, I = item.y;
      const int slot = g_item_slot[it];
      const int32_t* __restrict__ kv = g_kv_idx + g_row_ptr[h * p.nQ + I];
      const int64_t bh = (int64_t)bb * p.H + h;
      const unsigned char* kbase = reinterpret_cast<const unsigned char*>(p.k + bh * p.nK * BLK * D);
      const unsigned char* vbase = reinterpret_cast<const unsigned char*>(p.v + bh * p.nK * BLK * D);

      auto issue_loads = [&](int J, int buf) {
        const unsigned char* kt = kbase + (int64_t)J * C::TILE_BYTES;
        const unsigned char* vt = vbase + (int64_t)J * C::TILE_BYTES;
#pragma unroll
        for (int i = 0; i < C::LOADS; ++i) {
          const int dst = buf * C::TILE_BYTES + (i * C::NW + w) * 1024;
          __builtin_amdgcn_global_load_lds((const GLOBAL_PTR(void))(kt + k_src[i]), (LDS_PTR(void))(lds + K_OFF + dst), 16, 0, 0);
          __builtin_amdgcn_global_load_lds((const GLOBAL_PTR(void))(vt + v_src[i]), (LDS_PTR(void))(lds + V_OFF + dst), 16, 0, 0);
        }
      };

      issue_loads(kv[item.z], 0);

      // Q^T operands of this wave's 64 queries: lane (r, g) holds q[32*qt + r][16ks + 8g .. +7]
      const int q0 = 64 * wa;
      bf16x8 qreg[C::QT][C::KS_QK];
#pragma unroll
      for (int qt = 0; qt < C::QT; ++qt) {
        const uint16_t* qrow = p.q + (bh * p.nQ * BLK + (int64_t)I * BLK + q0 + 32 * qt + r) * D;
#pragma unroll
        for (int ks = 0; ks < C::KS_QK; ++ks)
          qreg[qt][ks] = as_bf16x8(*reinterpret_cast<const u32x4*>(qrow + 16 * ks + 8 * g));
      }

      f32x16 oacc[C::DT][C::QT];
#pragma unroll
      for (int dt = 0; dt < C::DT; ++dt)
#pragma unroll
        for (int qt = 0; qt < C::QT; ++qt)
#pragma unroll
          for (int i = 0; i < 16; ++i) oacc[dt][qt][i] = 0.f;
      float m_run[C::QT], l_run[C::QT];
#pragma unroll
      for (int qt = 0; qt < C::QT; ++qt) { m_run[qt] = -INFINITY; l_run[qt] = 0.f; }

      for (int j = item.z; j < item.w; ++j) {
        const int buf = (j - item.z) & 1;
        __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): this wave's copies of block j have landed
        __syncthreads();                      // ... and everybody's; all waves are done with block j-1
        if (j + 1 < item.w) issue_loads(kv[j + 1], buf ^ 1);

        const unsigned char* sK = lds + K_OFF + buf * C::TILE_BYTES;
        const unsigned char* sV = lds + V_OFF + buf * C::TILE_BYTES;

        // S^T = K Q^T : [KW keys of this wave] x [64 queries of this wave]
        f32x16 sacc[C::KTW][C::QT];
#pragma unroll
        for (int kt = 0; kt < C::KTW; ++kt)
#pragma unroll
          for (int qt = 0; qt < C::QT; ++qt)
#pragma unroll
            for (int i = 0; i < 16; ++i) sacc[kt][qt][i] = 0.f;
#pragma unroll
        for (int ks = 0; ks < C::KS_QK; ++ks) {
#pragma unroll
          for (int kt = 0; kt < C::KTW; ++kt) {
            const bf16x8 a = as_bf16x8(*reinterpret_cast<const u32x4*>(sK + k_rd[ks] + kt * 32 * C::ROW_BYTES));
#pragma unroll
            for (int qt = 0; qt < C::QT; ++qt)
              sacc[kt][qt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qreg[qt][ks], sacc[kt][qt], 0, 0, 0);
          }
        }

        // online softmax over this wave's keys (per query = per lane pair r, r+32)
#pragma unroll
        for (int qt = 0; qt < C::QT; ++qt) {
          float mx = sacc[0][qt][0];
#pragma unroll
          for (int kt = 0; kt < C::KTW; ++kt)
#pragma unroll
            for (int i = 0; i < 16; ++i) mx = fmaxf(mx, sacc[kt][qt][i]);
          mx = fmaxf(mx, xor32(mx));
          const float m_new = fmaxf(m_run[qt], mx);
          const float alpha = __builtin_amdgcn_exp2f((m_run[qt] - m_new) * c);
          const float mc = m_new * c;
          m_run[qt] = m_new;
          float lsum = 0.f;
#pragma unroll
          for (int kt = 0; kt < C::KTW; ++kt)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
              const float pe = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[kt][qt][i], c, -mc));
              sacc[kt][qt][i] = pe;
              lsum += pe;
            }
          l_run[qt] = l_run[qt] * alpha + lsum;
#pragma unroll
          for (int dt = 0; dt < C::DT; ++dt)
#pragma unroll
            for (int i = 0; i < 16; ++i) oacc[dt][qt][i] *= alpha;
        }

        // O^T += V^T P^T
#pragma unroll
        for (int ks = 0; ks < C::KS_PV; ++ks) {
          const int kt = ks >> 1, hf = ks & 1;
          bf16x8 bp[C::QT];
#pragma unroll
          for (int qt = 0; qt < C::QT; ++qt) {
            u32x4 pb;
            pb.x = pack_bf16x2(sacc[kt][qt][8 * hf + 0], sacc[kt][qt][8 * hf + 1]);
            pb.y = pack_bf16x2(sacc[kt][qt][8 * hf + 2], sacc[kt][qt][8 * hf + 3]);
            pb.z = pack_bf16x2(sacc[kt][qt][8 * hf + 4], sacc[kt][qt][8 * hf + 5]);
            pb.w = pack_bf16x2(sacc[kt][qt][8 * hf + 6], sacc[kt][qt][8 * hf + 7]);
            bp[qt] = as_bf16x8(pb);
          }
#pragma unroll
          for (int dt = 0; dt < C::DT; ++dt) {
            const unsigned char* va = sV + v_rd[dt] + ks * 16 * C::ROW_BYTES;
            const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_PTR(s16x4))(va));
            const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LDS_PTR(s16x4))(va + 8 * C::ROW_BYTES));
            const bf16x8 a = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
#pragma unroll
            for (int qt = 0; qt < C::QT; ++qt)
              oacc[dt][qt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, bp[qt], oacc[dt][qt], 0, 0, 0);
          }
        }
      }

      // ---- combine the two key halves: wave (a, c) finalises d-tiles [c*DT/2, (c+1)*DT/2) ----
      __syncthreads();   // every wave is done reading the K/V tiles: the buffers become the exchange area
      constexpr int HT = C::DT / 2;
      float* xo = reinterpret_cast<float*>(lds) + w * (C::QT * HT * 16 * 64);
      float* xs = reinterpret_cast<float*>(lds) + C::NW * (C::QT * HT * 16 * 64) + w * (C::QT * 2 * 64);
      const int pw = wa * C::NKH + (1 - wc);   // partner wave: same queries, other key half
      const float* yo = reinterpret_cast<const float*>(lds) + pw * (C::QT * HT * 16 * 64);
      const float* ys = reinterpret_cast<const float*>(lds) + C::NW * (C::QT * HT * 16 * 64) + pw * (C::QT * 2 * 64);
      const int64_t tok0 = bh * p.nQ * BLK + (int64_t)I * BLK + q0 + r;
      const int64_t ps = (int64_t)bb * p.n_slots + slot;

      // WC is this wave's key half as a compile-time constant, so that the accumulator tiles
      // are addressed with constant indices (they must stay in registers)
      auto finish = [&](auto wc_tag) {
        constexpr int WC = decltype(wc_tag)::value;
        float l_full[C::QT];
#pragma unroll
        for (int qt = 0; qt < C::QT; ++qt) {
          l_full[qt] = l_run[qt] + xor32(l_run[qt]);
          xs[(2 * qt + 0) * 64 + l] = m_run[qt];
          xs[(2 * qt + 1) * 64 + l] = l_full[qt];
#pragma unroll
          for (int hx = 0; hx < HT; ++hx)
#pragma unroll
            for (int i = 0; i < 16; ++i) xo[((qt * HT + hx) * 16 + i) * 64 + l] = oacc[(1 - WC) * HT + hx][qt][i];
        }
        __syncthreads();
#pragma unroll
        for (int qt = 0; qt < C::QT; ++qt) {
          const float mp = ys[(2 * qt + 0) * 64 + l], lp = ys[(2 * qt + 1) * 64 + l];
          const float mt = fmaxf(m_run[qt], mp);
          const float fs = __builtin_amdgcn_exp2f((m_run[qt] - mt) * c);
          const float fp = __builtin_amdgcn_exp2f((mp - mt) * c);
          const float lt = l_full[qt] * fs + lp * fp;
          const float inv = 1.0f / lt;
          const float fsi = fs * inv, fpi = fp * inv;
          const int64_t tok = tok0 + 32 * qt;
#pragma unroll
          for (int hx = 0; hx < HT; ++hx) {
            float res[16];
#pragma unroll
            for (int i = 0; i < 16; ++i)
              res[i] = oacc[WC * HT + hx][qt][i] * fsi + yo[((qt * HT + hx) * 16 + i) * 64 + l] * fpi;
            if (slot < 0) {
              uint16_t* orow = p.o + tok * D + 32 * (WC * HT + hx) + 4 * g;
#pragma unroll
              for (int i4 = 0; i4 < 4; ++i4) {
                u32x2 pk;
                pk.x = pack_bf16x2(res[4 * i4 + 0], res[4 * i4 + 1]);
                pk.y = pack_bf16x2(res[4 * i4 + 2], res[4 * i4 + 3]);
                *reinterpret_cast<u32x2*>(orow + 8 * i4) = pk;
              }
            } else {
              float* orow = p.part_o + (ps * BLK + q0 + 32 * qt + r) * D + 32 * (WC * HT + hx) + 4 * g;
#pragma unroll
              for (int i4 = 0; i4 < 4; ++i4) {
                f32x4 f = {res[4 * i4 + 0], res[4 * i4 + 1], res[4 * i4 + 2], res[4 * i4 + 3]};
                *reinterpret_cast<f32x4*>(orow + 8 * i4) = f;
              }
            }
          }
          if (WC == 0 && g == 0) {
            const float lse = mt * p.scale + __logf(lt);
            if (slot < 0) { if (p.lse != nullptr) p.lse[tok] = lse; }
            else p.part_lse[ps * BLK + q0 + 32 * qt + r] = lse;
          }
        }
      };
      if (wc == 0) finish(std::integral_constant<int, 0>{});
      else finish(std::integral_constant<int, 1>{});
      __syncthreads();   // exchange area fully read before the next item's copies overwrite it
      busy += wall_clock64() - t0;
    }
  }

  if (t == 0) {
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
// Grid: B * (n_split + n_empty) workgroups of 256 threads.
template <int D>
__global__ __launch_bounds__(256) void dbsp_fixup_kernel(const dbsp_fwd_params p, int blk) {
  const int per_b = p.n_split + p.n_empty;
  const int bb = blockIdx.x / per_b, e = blockIdx.x % per_b;
  const int n4 = blk * (D / 4);
  if (e < p.n_split) {
    const int4 sr = reinterpret_cast<const int4*>(p.split_rows)[e];
    const int row = sr.x, first = sr.y, nch = sr.z;
    const int h = row / p.nQ, I = row % p.nQ;
    const int64_t bh = (int64_t)bb * p.H + h;
    const int64_t ps0 = (int64_t)bb * p.n_slots + first;
    for (int x = threadIdx.x; x < n4; x += 256) {
      const int qloc = x / (D / 4), d4 = x % (D / 4);
      float mx = -INFINITY;
      for (int kx = 0; kx < nch; ++kx) mx = fmaxf(mx, p.part_lse[(ps0 + kx) * blk + qloc]);
      float tot = 0.f;
      for (int kx = 0; kx < nch; ++kx) tot += __expf(p.part_lse[(ps0 + kx) * blk + qloc] - mx);
      const float lse = mx + __logf(tot);
      f32x4 acc = {0.f, 0.f, 0.f, 0.f};
      for (int kx = 0; kx < nch; ++kx) {
        const float wgt = __expf(p.part_lse[(ps0 + kx) * blk + qloc] - lse);
        const f32x4 f = *reinterpret_cast<const f32x4*>(p.part_o + ((ps0 + kx) * blk + qloc) * D + 4 * d4);
        acc.x += wgt * f.x;  acc.y += wgt * f.y;  acc.z += wgt * f.z;  acc.w += wgt * f.w;
      }
      const int64_t tok = bh * p.nQ * blk + (int64_t)I * blk + qloc;
      u32x2 pk;
      pk.x = pack_bf16x2(acc.x, acc.y);
      pk.y = pack_bf16x2(acc.z, acc.w);
      *reinterpret_cast<u32x2*>(p.o + tok * D + 4 * d4) = pk;
      if (p.lse != nullptr && d4 == 0) p.lse[tok] = lse;
    }
  } else {
    const int row = p.empty_rows[e - p.n_split];
    const int h = row / p.nQ, I = row % p.nQ;
    const int64_t bh = (int64_t)bb * p.H + h;
    for (int x = threadIdx.x; x < n4; x += 256) {
      const int qloc = x / (D / 4), d4 = x % (D / 4);
      const int64_t tok = bh * p.nQ * blk + (int64_t)I * blk + qloc;
      *reinterpret_cast<u32x2*>(p.o + tok * D + 4 * d4) = u32x2{0u, 0u};
      if (p.lse != nullptr && d4 == 0) p.lse[tok] = -INFINITY;
    }
  }
}

template <int BLK, int D>
hipError_t launch_fwd(const dbsp_fwd_params& p, int P, hipStream_t stream) {
  using C = Cfg<BLK, D>;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&dbsp_fwd_kernel<BLK, D>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, C::LDS_BYTES);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  hipLaunchKernelGGL((dbsp_fwd_kernel<BLK, D>), dim3(P), dim3(C::NT), C::LDS_BYTES, stream, p, p.row_ptr, p.kv_idx,
                     reinterpret_cast<const int4*>(p.items), p.item_slot, p.part_ptr, p.part_items);
  return hipGetLastError();
}

}  // namespace

hipError_t dbsp_launch_fwd(const dbsp_fwd_params& p, int block, int d, int P, hipStream_t stream) {
  hipError_t e;
  if (block == 128 && d == 128) e = launch_fwd<128, 128>(p, P, stream);
  else if (block == 128 && d == 64) e = launch_fwd<128, 64>(p, P, stream);
  else if (block == 64 && d == 128) e = launch_fwd<64, 128>(p, P, stream);
  else if (block == 64 && d == 64) e = launch_fwd<64, 64>(p, P, stream);
  else return hipErrorInvalidValue;
  if (e != hipSuccess) return e;
  const int fix = p.B * (p.n_split + p.n_empty);
  if (fix > 0) {
    if (d == 128) hipLaunchKernelGGL((dbsp_fixup_kernel<128>), dim3(fix), dim3(256), 0, stream, p, block);
    else hipLaunchKernelGGL((dbsp_fixup_kernel<64>), dim3(fix), dim3(256), 0, stream, p, block);
    e = hipGetLastError();
  }
  return e;
}
