// dK / dV part of fcp_attn_bwd_step.
//
// Backward of O = softmax(scale Q K^T) V (paper Eq. 1, Sec. 3.1; causal mask, Sec. 4.3) for the key sets the
// ring steps bring (ring-style CP, Sec. 3.2).  With the merged LSE the probabilities of a step are recomputed
// exactly, P = exp(scale s - LSE), so each step adds its own share:
//   dV += P^T dO,   dS = P o (dO V^T - delta),   dK += scale dS^T Q,
// summed over the query heads of a KV head and over the query rows that see the key.
//
// gfx950 design
//   * persistent 512-thread blocks (8 wave64, one block per CU, two waves per SIMD) pull (key tile, KV head)
//     units from per-XCD counters; the list is sorted longest-first;
//   * a unit = 128 keys of one segment of one work item for one KV head, looping over the query heads of the
//     KV head and over the 32-row query blocks that see the tile.  Waves w and w+4 share a SIMD (measured) and
//     the SAME 32 keys, and split the work by ROLE so that each fits 256 registers:
//       wave w   ("P wave"):   S = Q K^T, P = exp2(c S - LSE log2 e) with the mask, dV^T += dO^T P;
//                              keeps K fragments and the dV^T accumulators, hands P (fp32) over through LDS;
//       wave w+4 ("dS wave"):  dP - delta = dO V^T with the accumulator started at -delta, dS = P o (dP - delta),
//                              dK^T += Q^T dS; keeps V fragments and the dK^T accumulators; runs ONE STEP BEHIND,
//                              so that the P it needs was written before the step's barrier;
//     on this chip the matrix and vector instructions of ONE wave hardly overlap while those of the two waves
//     of a SIMD do, so the pair keeps the matrix pipe busy while either of them is in its vector phase;
//   * Q, dO blocks (32 rows) and their row statistics stream through LDS in four stages filled by LDS-direct
//     buffer loads; the tiles are chunk-permuted so that both the row reads (A operands of S and dP) and the
//     transpose reads (A operands dO^T, Q^T of the accumulating contractions) run at the full LDS rate;
//   * S and dP come out as [query x key] with the key on the lane, which is exactly the B-operand layout of
//     dV^T += dO^T P and dK^T += Q^T dS;
//   * inside the matrix phases every LDS fragment is requested several MFMAs before its use;
//   * the result is added to the caller's fp32 accumulators once per unit: with plain load-add-store when the
//     scheduler found that no other item of the launch touches the same keys, otherwise with fp32 atomics.
#include "fcp_bwd.h"

namespace fcp {
namespace {

template <int D>
struct DkvCfg {
  static constexpr int BN = kBwdBN;                // 128 keys per unit (32 per wave pair)
  static constexpr int BM = kBwdBM;                // 32 query rows per step
  static constexpr int NWAVE = 8;
  using DT = DualTile<D>;
  static constexpr int TILE = DT::bytes(BM);       // one Q or dO block
  static constexpr int SLOT = 256;                 // one statistics slot: 64 floats (32 used)
  static constexpr int STAGE = 2 * TILE + NWAVE * SLOT;   // Q, dO, one statistics slot per wave (0: -LSE log2 e, 1: -delta)
  static constexpr int NSTAGE = 4;
  static constexpr int PBYTES = 32 * 32 * 4;       // one P block of a wave pair, fp32, lane-major
  static constexpr int POFF = NSTAGE * STAGE;      // P buffers: [pair][2]
  static constexpr int LDS_BYTES = POFF + 4 * 2 * PBYTES;
  static constexpr int NS = D / 16;                // MFMAs of one 32 x 32 block of S or dP
  static constexpr int NVA = D / 32;               // 32-channel blocks of dK^T / dV^T
  static constexpr int TINST = 2 * BM / DT::RPI;   // tile fill instructions per step (Q then dO)
  static constexpr int IPW = TINST / NWAVE;        // ... per wave
  static constexpr int FILLS = IPW + 1;            // ... plus the wave's statistics load
  static constexpr int kWaitFills = 0x0F70 | FILLS;
  static constexpr int kAhead = 4;                 // LDS fragments requested this many MFMAs ahead
  static_assert(TINST % NWAVE == 0 && FILLS < 16, "fill split");
};

template <int D>
__global__ __launch_bounds__(512, 1) void dkv_kernel(const BwdParams p) {
  using C = DkvCfg<D>;
  using DT = typename C::DT;
  extern __shared__ __attribute__((aligned(256))) unsigned char smem[];
  __shared__ int32_t s_next_unit;
  __shared__ int32_t s_rec[16];

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int role = wave >> 2;                     // 0: P wave, 1: dS wave (one step behind)
  const int pw = wave & 3;                        // key group of the pair: keys 32 pw .. 32 pw + 31
  const int l32 = lane & 31, g2 = lane >> 5;
  const int G = p.hq / p.hkv;
  const uint32_t lds0 = lds_offset(smem);
  const bool per_xcd = (p.hkv % kNumXcd) == 0;
  const int xcd = per_xcd ? (int)(blockIdx.x % kNumXcd) : 0;
  const int kvh_here = per_xcd ? p.hkv / kNumXcd : p.hkv;
  UnitQueue uq;
  uq.init(p.hdr, p.tiles, xcd, kvh_here, &s_next_unit, s_rec);

  // ---- per-lane constants -----------------------------------------------------------------
  const int q_row_bytes = p.hq * D * 2;
  // LDS-direct fills: tile instruction j (0 .. TINST-1; the first half fills Q, the second dO) covers block rows
  // RPI (j % (TINST/2)) ..; wave w issues instructions w, w + 8, ..
  int tfill[C::IPW];
#pragma unroll
  for (int i = 0; i < C::IPW; ++i) {
    const int j = (wave + C::NWAVE * i) % (C::TINST / 2);
    const int row = DT::RPI * j + lane / DT::CPR;
    tfill[i] = row * q_row_bytes + (((lane % DT::CPR) ^ DT::key(row)) << 4);
  }
  // row fragments (A operands of S = Q K^T, dP = dO V^T): lane reads block row l32, chunk 2 ks + g2
  int rowaddr[C::NS];
#pragma unroll
  for (int ks = 0; ks < C::NS; ++ks) rowaddr[ks] = tile_off<DT>(l32, 2 * ks + g2);
  // transposed fragments (A operands dO^T, Q^T [channel x query]; k-slots = query rows 16 t + {4 g2 + [0,4),
  // 8 + 4 g2 + [0,4)}): inside a 16-lane block lane i supplies the address of block row (i / 4), channels
  // 4 (i % 4) + [0,4); block b covers channels 16 (b % 2) + [0,16) for row group b / 2
  int traddr[2][C::NVA];
  {
    const int row0 = 4 * g2 + ((lane & 15) >> 2);
    const int chunk0 = 2 * ((lane >> 4) & 1) + ((lane & 3) >> 1);
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
      for (int db = 0; db < C::NVA; ++db) traddr[h][db] = tile_off<DT>(row0 + 8 * h, 4 * db + chunk0) + 8 * (lane & 1);
  }
  unsigned char* const pbuf = smem + C::POFF + pw * (2 * C::PBYTES) + lane * 16;   // lane-major: 4 x 16 bytes per lane

  PhaseTimer pt;
  pt.begin();
  for (;;) {
    const int unit = uq.current(&s_next_unit);
    if (unit >= uq.n_units) break;
    const KTile t = read_record<KTile>(s_rec);
    const int kvh = xcd * kvh_here + unit % kvh_here;
    uq.prefetch();

    const bool exclusive = (t.flags & kFlagSeg0Exclusive) != 0;
    const int n_keys = t.n_keys;                               // >= 1 by construction
    const int my_key = 32 * pw + l32;
    const int my_key_ld = min(my_key, n_keys - 1);
    const bool my_key_valid = my_key < n_keys;
    const bool pair_has_keys = 32 * pw < n_keys;
    const int64_t kv_row0 = t.kv_row0;

    // query blocks that see the tile: from the block holding the first row at or after the tile's first key
    const int first_row = max(0, t.k_pos0 - t.q_seq_start);
    const int qb0 = first_row / C::BM;
    const int nqb = (t.q_len + C::BM - 1) / C::BM - qb0;       // query blocks per head, >= 1
    const int n_iter = nqb * G;

    // own-key fragments, B operand (lane = key column): K for the P wave, V for the dS wave
    bf16x8 kvf[C::NS];
    {
      const uint16_t* src = role == 0 ? p.k : p.v;
      const int64_t off = ((kv_row0 + my_key_ld) * p.hkv + kvh) * D + 8 * g2;
#pragma unroll
      for (int ks = 0; ks < C::NS; ++ks) kvf[ks] = *reinterpret_cast<const bf16x8*>(src + off + 16 * ks);
    }

    // ---- fills ---------------------------------------------------------------------------------
    // Step s = (query head s / nqb of the KV head, query block qb0 + s % nqb).  The running state below names
    // the NEXT step to be filled; steps are filled strictly in order.  Rows past the item's last row lie
    // outside the resources' range and arrive as zeros.  Every call issues exactly FILLS loads (past the last
    // step they fall outside the range), which the vmcnt waits rely on.
    const int q_bytes = (t.q_len - 1) * q_row_bytes + D * 2;
    const int64_t plane = (int64_t)p.hq * p.tq;               // floats per statistics plane
    int f_head = kvh * G, f_left = nqb, f_heads_left = G;
    int f_soff = qb0 * C::BM * q_row_bytes, f_ssoff = qb0 * C::BM * 4;
    auto f_resources = [&](bool live, i32x4& rq, i32x4& rdo, i32x4& rst) {
      rq = buffer_rsrc(p.q + ((int64_t)t.q_local_off * p.hq + f_head) * D, live ? q_bytes : 0);
      rdo = buffer_rsrc(p.d_o + ((int64_t)t.q_local_off * p.hq + f_head) * D, live ? q_bytes : 0);
      rst = buffer_rsrc(p.stats + (wave & 1) * plane + (int64_t)f_head * p.tq + t.q_local_off, live ? t.q_len * 4 : 0);
    };
    i32x4 f_rq, f_rdo, f_rst;
    f_resources(true, f_rq, f_rdo, f_rst);
    uint32_t f_dst = lds0;
    auto fill_next = [&]() {
      if (f_left == 0) {          // next head of the group (or past the end: empty resources)
        --f_heads_left;
        ++f_head;
        f_left = nqb;
        f_soff = qb0 * C::BM * q_row_bytes;
        f_ssoff = qb0 * C::BM * 4;
        f_resources(f_heads_left > 0, f_rq, f_rdo, f_rst);
      }
#pragma unroll
      for (int i = 0; i < C::IPW; ++i) {
        const int j = wave + C::NWAVE * i;                       // wave-uniform
        const bool is_do = j >= C::TINST / 2;
        const uint32_t d = f_dst + (is_do ? C::TILE : 0) + DT::row_base(DT::RPI * (j % (C::TINST / 2)));
        lds_fill_b128(is_do ? f_rdo : f_rq, d, tfill[i], f_soff);
      }
      lds_fill_b32(f_rst, f_dst + 2 * C::TILE + wave * C::SLOT, lane * 4, f_ssoff);
      --f_left;
      f_soff += C::BM * q_row_bytes;
      f_ssoff += C::BM * 4;
      f_dst += C::STAGE;
      if (f_dst >= lds0 + C::NSTAGE * C::STAGE) f_dst -= C::NSTAGE * C::STAGE;
    };
    fill_next();
    fill_next();

    f32x16 acc[C::NVA];          // dV^T (P wave) or dK^T (dS wave) [channel x own key]
#pragma unroll
    for (int db = 0; db < C::NVA; ++db) acc[db] = zero16();

    // ---- the steps -------------------------------------------------------------------------------
    // Iteration `it`: the P waves work on step it, the dS waves on step it - 1.  At its top every wave has waited
    // for all its fills but the newest batch (step it + 1) and met the others: the blocks of steps it - 1 and it
    // are in LDS, P of step it - 1 is in its buffer, and stage (it + 2) % 4, last read by the dS waves in
    // iteration it - 1, is free for the fills of step it + 2.
    int qb = qb0;                                            // query block of this wave's current step
    for (int it = 0; it <= n_iter; ++it) {
      pt.mark(0);
      __builtin_amdgcn_s_waitcnt(C::kWaitFills);
      __syncthreads();
      pt.mark(1);
      fill_next();
      const int sidx = it - role;                            // this wave's step
      if (sidx < 0 || sidx >= n_iter) continue;
      const int row0 = qb * C::BM;
      const int q_pos0 = t.q_seq_start + row0;
      const int rows_here = min(C::BM, t.q_len - row0);
      if (++qb == qb0 + nqb) qb = qb0;
      // pair-uniform: nothing to contribute if the pair has no key in the tile or all its keys lie after the
      // block's rows
      if (!pair_has_keys || t.k_pos0 + 32 * pw > q_pos0 + rows_here - 1) continue;

      const unsigned char* qs = smem + (sidx & (C::NSTAGE - 1)) * C::STAGE;
      const unsigned char* dos = qs + C::TILE;
      const float* stat = reinterpret_cast<const float*>(dos + C::TILE);   // slot 0: -LSE log2 e; slot 1: -delta
      unsigned char* const pslot = pbuf + (sidx & 1) * C::PBYTES;
      const unsigned char* const rtile = role == 0 ? qs : dos;             // tile read by rows
      const unsigned char* const ttile = role == 0 ? dos : qs;             // tile read transposed
      pt.mark(2);

      // Phase 1: S = Q K^T (P wave) or dP - delta = dO V^T - delta (dS wave) [32 rows x 32 own keys]; register i
      // of the result is block row 8 (i/4) + 4 g2 + i%4, so the four row statistics a lane needs per group of
      // four registers are contiguous
      f32x16 sacc;
      f32x4 nl[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) nl[j] = *reinterpret_cast<const f32x4*>(stat + role * (C::SLOT / 4) + 8 * j + 4 * g2);
      if (role == 0) sacc = zero16();
      else {
#pragma unroll
        for (int i = 0; i < 16; ++i) sacc[i] = nl[i / 4][i % 4];
      }
      {
        bf16x8 fr[C::NS];
        auto request = [&](int x) { if (x < C::NS) fr[x] = *reinterpret_cast<const bf16x8*>(rtile + rowaddr[x]); };
#pragma unroll
        for (int x = 0; x < C::kAhead; ++x) request(x);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int x = 0; x < C::NS; ++x) {
          sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[x], kvf[x], sacc, 0, 0, 0);
          request(x + C::kAhead);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
      // Phase 2 (vector): P wave: P = exp2(c S - LSE log2 e) with the mask, stored for the partner;
      //                   dS wave: dS = P o (dP - delta) with the partner's P
      bf16x8 bop[2];           // B operand of phase 3: P or dS, k-step tt covers block rows 16 tt .. 16 tt + 15
      if (role == 0) {
        const bool need_mask = (t.k_pos0 + 32 * pw + 31 > q_pos0) || (32 * pw + 32 > n_keys) || (rows_here < C::BM);
        const int lo = (my_key_valid ? t.k_pos0 + my_key - q_pos0 : 1 << 20) - 4 * g2;   // first row (minus 4 g2) that sees the key
        const int hi = rows_here - 4 * g2;
        f32x4 pr[4];
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          float e = __builtin_amdgcn_exp2f(fmaf(sacc[i], p.scale_log2, nl[i / 4][i % 4]));
          if (need_mask) {
            const int c = 8 * (i / 4) + (i % 4);
            if (c < lo || c >= hi) e = 0.f;
          }
          pr[i / 4][i % 4] = e;
          bop[i / 8][i % 8] = (__bf16)e;
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) *reinterpret_cast<f32x4*>(pslot + j * 1024) = pr[j];
      } else {
        f32x4 pr[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) pr[j] = *reinterpret_cast<const f32x4*>(pslot + j * 1024);
#pragma unroll
        for (int i = 0; i < 16; ++i) bop[i / 8][i % 8] = (__bf16)(pr[i / 4][i % 4] * sacc[i]);
      }
      pt.mark(3);
      // Phase 3: dV^T += dO^T P (P wave) or dK^T += Q^T dS (dS wave)
      {
        constexpr int N = 2 * C::NVA;
        bf16x8 fr[N];
        auto request = [&](int x) {
          if (x < N) {
            const unsigned char* b0 = ttile + (x / C::NVA) * (16 * DT::row_base(1));
            fr[x] = tr_read_8(b0 + traddr[0][x % C::NVA], b0 + traddr[1][x % C::NVA]);
          }
        };
#pragma unroll
        for (int x = 0; x < C::kAhead; ++x) request(x);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int x = 0; x < N; ++x) {
          acc[x % C::NVA] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[x], bop[x / C::NVA], acc[x % C::NVA], 0, 0, 0);
          request(x + C::kAhead);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
      pt.mark(4);
    }

    // epilogue: dV^T or dK^T [channel x own key] -> pool accumulators
    if (my_key_valid) {
      float* dst = (role == 0 ? p.dv : p.dk) + ((kv_row0 + my_key) * p.hkv + kvh) * D + 4 * g2;
      const float mul = role == 0 ? 1.f : p.scale;
#pragma unroll
      for (int db = 0; db < C::NVA; ++db)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          const int c = 32 * db + 8 * r4;
          if (exclusive) {
            f32x4 a = *reinterpret_cast<f32x4*>(dst + c);
#pragma unroll
            for (int e = 0; e < 4; ++e) a[e] += acc[db][4 * r4 + e] * mul;
            *reinterpret_cast<f32x4*>(dst + c) = a;
          } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) unsafeAtomicAdd(dst + c + e, acc[db][4 * r4 + e] * mul);
          }
        }
    }
    uq.advance(&s_next_unit, s_rec);   // barrier: the LDS stages are free for the next unit's fills
  }
  pt.end(p.hdr);
}

// Row statistics in the form the kernels consume: plane 0 = -LSE log2 e (-inf for a row without keys, so that
// its probabilities vanish), plane 1 = -delta.
__global__ __launch_bounds__(256) void row_stats_kernel(const float* __restrict__ lse, const float* __restrict__ delta,
                                                        int64_t n, float* __restrict__ stats) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
    const float l = lse[i];
    stats[i] = l == -INFINITY ? -INFINITY : -l * kLog2e;
    stats[n + i] = -delta[i];
  }
}

}  // namespace

int launch_row_stats(const float* lse, const float* delta, int64_t n, float* stats, hipStream_t stream) {
  if (n <= 0) return FCP_OK;
  int64_t blocks = (n + 255) / 256;
  if (blocks > 2048) blocks = 2048;
  hipLaunchKernelGGL(row_stats_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, lse, delta, n, stats);
  FCP_HIP_CHECK(hipGetLastError());
  return FCP_OK;
}

int launch_dkv(const BwdParams& p, int head_dim, int64_t units, int n_cu, hipStream_t stream) {
  int64_t blocks = n_cu;                               // one 512-thread block per CU
  if (blocks > units) blocks = (units + 7) / 8 * 8;   // a multiple of the XCD count
  if (blocks < 8) blocks = 8;
  static bool attr_done[2] = {false, false};
  if (head_dim == 128) {
    if (!attr_done[0]) {
      FCP_HIP_CHECK(hipFuncSetAttribute((const void*)dkv_kernel<128>, hipFuncAttributeMaxDynamicSharedMemorySize, DkvCfg<128>::LDS_BYTES));
      attr_done[0] = true;
    }
    hipLaunchKernelGGL(dkv_kernel<128>, dim3((unsigned)blocks), dim3(512), DkvCfg<128>::LDS_BYTES, stream, p);
  } else {
    if (!attr_done[1]) {
      FCP_HIP_CHECK(hipFuncSetAttribute((const void*)dkv_kernel<64>, hipFuncAttributeMaxDynamicSharedMemorySize, DkvCfg<64>::LDS_BYTES));
      attr_done[1] = true;
    }
    hipLaunchKernelGGL(dkv_kernel<64>, dim3((unsigned)blocks), dim3(512), DkvCfg<64>::LDS_BYTES, stream, p);
  }
  FCP_HIP_CHECK(hipGetLastError());
  return FCP_OK;
}

}  // namespace fcp
