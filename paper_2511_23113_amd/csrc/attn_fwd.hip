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
// Register/LDS layout (wave = 64 lanes, lane = 32*g + r):
//   * The products are formed transposed, S^T = K Q^T and O^T = V^T P^T, with
//     v_mfma_f32_32x32x16_bf16.  Each wave owns 32 query columns; lane r holds query r, so the
//     softmax statistics m, l are per-lane scalars and reductions over keys stay inside a lane
//     (plus one exchange with lane r+32).
//   * S^T's accumulator registers 8h..8h+7 of a 32-key tile hold, in lane group g, the keys
//     16h + {4g..4g+3, 8+4g..8+4g+3}; packed to bf16 they ARE the B operand of the PV product
//     for that 16-key step, provided V^T's A operand uses the same key order.  V is therefore
//     stored in LDS transposed ([d][key]) with the two middle 4-key groups of every 16 keys
//     swapped, so that one 16-byte LDS read yields the matching A operand.
//   * K is stored row-major in LDS; rows are padded by 16 bytes so that the 16-byte operand
//     reads of 16 consecutive lanes fall into distinct banks.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "fwd_params.hpp"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) {
  f32x2 f = {a, b};
  bf16x2 h = __builtin_convertvector(f, bf16x2);  // round-to-nearest-even
  return __builtin_bit_cast(uint32_t, h);
}

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 u) { return __builtin_bit_cast(bf16x8, u); }

__device__ __forceinline__ float xor32(float x) { return __shfl_xor(x, 32, 64); }

template <int BLK, int D>
struct Cfg {
  static constexpr int NW = BLK / 32;       // waves; each owns 32 query columns
  static constexpr int NT = NW * 64;        // threads
  static constexpr int KT = BLK / 32;       // 32-key tiles per KV block
  static constexpr int DT = D / 32;         // 32-wide tiles of the head dim
  static constexpr int KS_QK = D / 16;      // k-steps of K Q^T
  static constexpr int KS_PV = BLK / 16;    // k-steps of V^T P^T
  static constexpr int KSTR = D + 8;        // LDS row stride of K   (elements)
  static constexpr int VSTR = BLK + 8;      // LDS row stride of V^T (elements)
  static constexpr int K_CH = (BLK * D / 8) / NT;            // 16-byte chunks of K per thread
  static constexpr int V_SUB = ((BLK / 4) * (D / 4)) / NT;   // 4x4 sub-blocks of V per thread
  static constexpr int LDS_BYTES = (BLK * KSTR + D * VSTR) * 2;
};

template <int BLK, int D>
__global__ __launch_bounds__(BLK * 2) void dbsp_fwd_kernel(const dbsp_fwd_params p) {
  using C = Cfg<BLK, D>;
  extern __shared__ __attribute__((aligned(16))) uint16_t lds[];
  uint16_t* sK = lds;
  uint16_t* sVt = lds + BLK * C::KSTR;

  const int t = threadIdx.x;
  const int w = t >> 6, l = t & 63, r = l & 31, g = l >> 5;
  const int part = blockIdx.x;
  const float c = p.scale_log2;

  uint64_t busy = 0;

  const int it_begin = p.part_ptr[part], it_end = p.part_ptr[part + 1];
  for (int bb = 0; bb < p.B; ++bb) {
    for (int ii = it_begin; ii < it_end; ++ii) {
      const uint64_t t0 = wall_clock64();
      const int it = p.part_items[ii];
      const int4 item = reinterpret_cast<const int4*>(p.items)[it];
      const int h = item.x, I = item.y;
      const int slot = p.item_slot[it];
      const int32_t* kv = p.kv_idx + p.row_ptr[h * p.nQ + I];
      const int64_t bh = (int64_t)bb * p.H + h;
      const uint16_t* kbase = p.k + bh * p.nK * BLK * D;
      const uint16_t* vbase = p.v + bh * p.nK * BLK * D;

      // Q^T operand of this wave's 32 queries: lane (r, g) holds q[r][16ks + 8g .. +7]
      const int qloc = 32 * w + r;
      const uint16_t* qrow = p.q + (bh * p.nQ * BLK + (int64_t)I * BLK + qloc) * D;
      bf16x8 qreg[C::KS_QK];
#pragma unroll
      for (int ks = 0; ks < C::KS_QK; ++ks)
        qreg[ks] = as_bf16x8(*reinterpret_cast<const u32x4*>(qrow + 16 * ks + 8 * g));

      f32x16 oacc[C::DT];
#pragma unroll
      for (int dt = 0; dt < C::DT; ++dt)
#pragma unroll
        for (int i = 0; i < 16; ++i) oacc[dt][i] = 0.f;
      float m_run = -INFINITY, l_run = 0.f;

      u32x4 kreg[C::K_CH];
      u32x2 vreg[C::V_SUB][4];
      auto prefetch = [&](int J) {
        const uint16_t* kt = kbase + (int64_t)J * BLK * D;
        const uint16_t* vt = vbase + (int64_t)J * BLK * D;
#pragma unroll
        for (int i = 0; i < C::K_CH; ++i) {
          const int ch = t + i * C::NT;
          kreg[i] = *reinterpret_cast<const u32x4*>(kt + ch * 8);  // chunk ch = row*(D/8) + col8: contiguous
        }
#pragma unroll
        for (int i = 0; i < C::V_SUB; ++i) {
          const int s = t + i * C::NT;
          const int dq = s % (D / 4), kq = s / (D / 4);
#pragma unroll
          for (int rr = 0; rr < 4; ++rr)
            vreg[i][rr] = *reinterpret_cast<const u32x2*>(vt + (4 * kq + rr) * D + 4 * dq);
        }
      };

      prefetch(kv[item.z]);
      for (int j = item.z; j < item.w; ++j) {
        __syncthreads();  // every wave is done reading the previous tile
#pragma unroll
        for (int i = 0; i < C::K_CH; ++i) {
          const int ch = t + i * C::NT;
          const int row = ch / (D / 8), col8 = ch % (D / 8);
          *reinterpret_cast<u32x4*>(sK + row * C::KSTR + col8 * 8) = kreg[i];
        }
#pragma unroll
        for (int i = 0; i < C::V_SUB; ++i) {
          const int s = t + i * C::NT;
          const int dq = s % (D / 4), kq = s / (D / 4);
          // key quad kq sits at quad position {0,2,1,3}[kq % 4] of its 16-key group
          const int q4 = kq & 3;
          const int pos = (kq >> 2) * 16 + (((q4 & 1) << 1) | (q4 >> 1)) * 4;
          const u32x2 r0 = vreg[i][0], r1 = vreg[i][1], r2 = vreg[i][2], r3 = vreg[i][3];
          u32x2 c0, c1, c2, c3;  // column cc of the 4x4 block = 4 keys of one d index
          c0.x = (r0.x & 0xffffu) | (r1.x << 16);  c0.y = (r2.x & 0xffffu) | (r3.x << 16);
          c1.x = (r0.x >> 16) | (r1.x & 0xffff0000u);  c1.y = (r2.x >> 16) | (r3.x & 0xffff0000u);
          c2.x = (r0.y & 0xffffu) | (r1.y << 16);  c2.y = (r2.y & 0xffffu) | (r3.y << 16);
          c3.x = (r0.y >> 16) | (r1.y & 0xffff0000u);  c3.y = (r2.y >> 16) | (r3.y & 0xffff0000u);
          uint16_t* dst = sVt + (4 * dq) * C::VSTR + pos;
          *reinterpret_cast<u32x2*>(dst) = c0;
          *reinterpret_cast<u32x2*>(dst + C::VSTR) = c1;
          *reinterpret_cast<u32x2*>(dst + 2 * C::VSTR) = c2;
          *reinterpret_cast<u32x2*>(dst + 3 * C::VSTR) = c3;
        }
        __syncthreads();
        if (j + 1 < item.w) prefetch(kv[j + 1]);  // global loads fly while this tile is computed

        // S^T = K Q^T : [BLK keys] x [32 queries of this wave]
        f32x16 sacc[C::KT];
#pragma unroll
        for (int kt = 0; kt < C::KT; ++kt)
#pragma unroll
          for (int i = 0; i < 16; ++i) sacc[kt][i] = 0.f;
#pragma unroll
        for (int ks = 0; ks < C::KS_QK; ++ks) {
#pragma unroll
          for (int kt = 0; kt < C::KT; ++kt) {
            const bf16x8 a = as_bf16x8(*reinterpret_cast<const u32x4*>(sK + (32 * kt + r) * C::KSTR + 16 * ks + 8 * g));
            sacc[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qreg[ks], sacc[kt], 0, 0, 0);
          }
        }

        // online softmax over the keys of this tile (per query = per lane pair r, r+32)
        float mx = sacc[0][0];
#pragma unroll
        for (int kt = 0; kt < C::KT; ++kt)
#pragma unroll
          for (int i = 0; i < 16; ++i) mx = fmaxf(mx, sacc[kt][i]);
        mx = fmaxf(mx, xor32(mx));
        const float m_new = fmaxf(m_run, mx);
        const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * c);
        const float mc = m_new * c;
        m_run = m_new;
        float lsum = 0.f;
#pragma unroll
        for (int kt = 0; kt < C::KT; ++kt)
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            const float pe = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[kt][i], c, -mc));
            sacc[kt][i] = pe;
            lsum += pe;
          }
        l_run = l_run * alpha + lsum;
#pragma unroll
        for (int dt = 0; dt < C::DT; ++dt)
#pragma unroll
          for (int i = 0; i < 16; ++i) oacc[dt][i] *= alpha;

        // O^T += V^T P^T
#pragma unroll
        for (int ks = 0; ks < C::KS_PV; ++ks) {
          const int kt = ks >> 1, hf = ks & 1;
          u32x4 pb;
          pb.x = pack_bf16x2(sacc[kt][8 * hf + 0], sacc[kt][8 * hf + 1]);
          pb.y = pack_bf16x2(sacc[kt][8 * hf + 2], sacc[kt][8 * hf + 3]);
          pb.z = pack_bf16x2(sacc[kt][8 * hf + 4], sacc[kt][8 * hf + 5]);
          pb.w = pack_bf16x2(sacc[kt][8 * hf + 6], sacc[kt][8 * hf + 7]);
          const bf16x8 bp = as_bf16x8(pb);
#pragma unroll
          for (int dt = 0; dt < C::DT; ++dt) {
            const bf16x8 a = as_bf16x8(*reinterpret_cast<const u32x4*>(sVt + (32 * dt + r) * C::VSTR + 16 * ks + 8 * g));
            oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, bp, oacc[dt], 0, 0, 0);
          }
        }
      }

      // epilogue: O / l, LSE = scale*m + ln l
      const float l_tot = l_run + xor32(l_run);
      const float inv = 1.0f / l_tot;
      const float lse = m_run * p.scale + __logf(l_tot);
      if (slot < 0) {
        uint16_t* orow = p.o + (bh * p.nQ * BLK + (int64_t)I * BLK + qloc) * D;
#pragma unroll
        for (int dt = 0; dt < C::DT; ++dt)
#pragma unroll
          for (int i4 = 0; i4 < 4; ++i4) {
            u32x2 pk;
            pk.x = pack_bf16x2(oacc[dt][4 * i4 + 0] * inv, oacc[dt][4 * i4 + 1] * inv);
            pk.y = pack_bf16x2(oacc[dt][4 * i4 + 2] * inv, oacc[dt][4 * i4 + 3] * inv);
            *reinterpret_cast<u32x2*>(orow + 32 * dt + 8 * i4 + 4 * g) = pk;
          }
        if (p.lse != nullptr && g == 0) p.lse[bh * p.nQ * BLK + (int64_t)I * BLK + qloc] = lse;
      } else {
        const int64_t ps = (int64_t)bb * p.n_slots + slot;
        float* orow = p.part_o + (ps * BLK + qloc) * D;
#pragma unroll
        for (int dt = 0; dt < C::DT; ++dt)
#pragma unroll
          for (int i4 = 0; i4 < 4; ++i4) {
            f32x4 f;
            f.x = oacc[dt][4 * i4 + 0] * inv;  f.y = oacc[dt][4 * i4 + 1] * inv;
            f.z = oacc[dt][4 * i4 + 2] * inv;  f.w = oacc[dt][4 * i4 + 3] * inv;
            *reinterpret_cast<f32x4*>(orow + 32 * dt + 8 * i4 + 4 * g) = f;
          }
        if (g == 0) p.part_lse[ps * BLK + qloc] = lse;
      }
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
  hipLaunchKernelGGL((dbsp_fwd_kernel<BLK, D>), dim3(P), dim3(C::NT), C::LDS_BYTES, stream, p);
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
