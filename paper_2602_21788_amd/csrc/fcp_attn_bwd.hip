// fcp_attn_bwd_step: gradient contributions of one CP rank for its ring steps.
//
// Backward of O = softmax(scale Q K^T) V (paper Eq. 1, Sec. 3.1; causal mask, Sec. 4.3) for
// the key sets the ring steps bring (ring-style CP, Sec. 3.2).  With the merged LSE the
// probabilities of a step are recomputed exactly, P = exp(scale s - LSE), so each step adds
// its own share:  dV += P^T dO,  dS = P o (dO V^T - delta),  dQ += scale dS K,  dK += scale dS^T Q.
//
// gfx950 design
//   * persistent 256-thread blocks pull (key tile, head) units, longest first;
//   * a unit = 128 keys of one segment of one work item for one query head; wave w owns keys
//     32w..32w+31: their K and V fragments live in registers for the whole unit and so do the
//     fp32 accumulators dK^T, dV^T [channel x own key];
//   * the loop runs over 32-row query blocks that can see the tile; Q and dO blocks are staged
//     in LDS (double buffered, next block's global loads in flight during compute);
//   * S = Q K^T and dP = dO V^T are produced as [query x key] with the key on the lane, so
//     P and dS are directly the B operands of dV^T += dO^T P and dK^T += Q^T dS, whose A
//     operands (dO^T, Q^T) come from the row-major LDS tiles by transpose reads;
//   * dQ needs the contraction over keys: dS goes once through LDS, then wave w computes the
//     [32 rows x 32 channels] slice w of dS K with K^T fragments kept in registers, and adds it
//     to the fp32 accumulator with 128-byte-contiguous hardware atomics;
//   * dK/dV are added to the pool accumulators once per unit (fp32 atomics), which also sums
//     the query heads of a KV head and the ring steps.
#include "fcp_internal.h"

namespace fcp {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

struct BwdParams {
  const uint16_t* q;
  const uint16_t* k;
  const uint16_t* v;
  const uint16_t* d_o;
  const float* lse;
  const float* delta;
  const int32_t* cu;
  const fcp_work_desc* work;
  const SchedHeader* hdr_ro;
  SchedHeader* hdr;
  const Tile* tiles;
  float* dq;
  float* dk;
  float* dv;
  int32_t tq, hq, hkv;
  float scale, scale_log2;
};

constexpr float kLog2e = 1.4426950408889634f;

template <int D>
struct BwdCfg {
  static constexpr int BN = kBwdBN;                // 128 keys per unit
  static constexpr int BM = kBwdBM;                // 32 query rows per inner step
  static constexpr int RSTRIDE = D * 2 + 64;       // Q/dO/K rows in LDS (bytes): serves b128 row reads
                                                   // (stride = 64 mod 256) and 4-row transpose reads
  static constexpr int KBYTES = BN * RSTRIDE;      // staged K tile (for the K^T fragments of dQ)
  static constexpr int QBYTES = BM * RSTRIDE;      // one Q or dO block
  static constexpr int SSTRIDE = BN * 2 + 16;      // dS rows [query][key] bf16
  static constexpr int SBYTES = BM * SSTRIDE;
  static constexpr int STAT_BYTES = 2 * BM * 4;    // LSE (log2 units) and delta of the block
  static constexpr int STAGE = 2 * QBYTES + STAT_BYTES;
  static constexpr int OFF_STAGE = KBYTES;
  static constexpr int OFF_DS = KBYTES + 2 * STAGE;
  static constexpr int LDS_BYTES = OFF_DS + SBYTES;
  static constexpr int CPR = D * 2 / 16;           // 16-byte pieces per row
  static constexpr int QPT = BM * CPR / 256;       // pieces per thread per tensor (2 for D=128, 1 for D=64)
};

__device__ inline bf16x8 tr_read_8(const unsigned char* p0, int row_stride4) {
  // two 4-row transpose reads -> 8 k-slots; rows p0 + [0,4) and p0 + row_stride4 bytes + [0,4)
  const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(p0));
  const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(p0 + row_stride4));
  return __builtin_shufflevector(__builtin_bit_cast(bf16x4, lo), __builtin_bit_cast(bf16x4, hi), 0, 1, 2, 3, 4, 5, 6, 7);
}

template <int D>
__global__ __launch_bounds__(256, 1) void bwd_kernel(const BwdParams p) {
  using C = BwdCfg<D>;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  __shared__ int32_t s_unit;

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, g2 = lane >> 5;
  const int G = p.hq / p.hkv;
  const bool per_xcd = (p.hq % kNumXcd) == 0;
  const int xcd = per_xcd ? (int)(blockIdx.x % kNumXcd) : 0;
  const int heads_here = per_xcd ? p.hq / kNumXcd : p.hq;
  const int n_units = p.hdr_ro->n_tiles * heads_here;

  // transpose-read lane geometry (see ds_read_b64_tr_b16): inside a 16-lane block the lane
  // addresses row (l%16)/4, 4 channels at 4*(l%4); blocks alternate channel halves, g2 picks rows
  const int tr_row = (lane & 15) >> 2;
  const int tr_col = 16 * ((lane >> 4) & 1) + 4 * (lane & 3);

  for (;;) {
    if (tid == 0) s_unit = atomicAdd(&p.hdr->counter[xcd], 1);
    __syncthreads();
    const int unit = __builtin_amdgcn_readfirstlane(s_unit);
    __syncthreads();
    if (unit >= n_units) break;
    const int tile_i = unit / heads_here;
    const int head = xcd * heads_here + unit % heads_here;
    const int kvh = head / G;
    const Tile tile = p.tiles[tile_i];
    const fcp_work_desc w = p.work[tile.work];
    const int seg = tile.idx >> 24, kt = tile.idx & 0xffffff;

    // keys of the unit
    const int vis_len = max(0, min(w.k_len[seg], w.q_seq_start + w.q_len - 1 - w.k_seq_start[seg] + 1));
    const int key0 = kt * C::BN;                               // first key (index in the segment)
    const int n_keys = min(C::BN, vis_len - key0);             // >= 1 by construction
    const int k_pos0 = w.k_seq_start[seg] + key0;
    const int64_t kv_row0 = (int64_t)p.cu[w.seq] + w.k_seq_start[seg] + key0;
    const int my_key = 32 * wave + l32;                        // key column this lane owns
    const int my_key_ld = min(my_key, n_keys - 1);
    const int my_k_pos = k_pos0 + my_key;
    const bool my_key_valid = my_key < n_keys;

    // query blocks that can see the tile
    const int first_row = max(0, k_pos0 - w.q_seq_start);
    const int qb0 = first_row / C::BM;
    const int qb1 = (w.q_len + C::BM - 1) / C::BM;

    // ---- one-time: K tile -> LDS (for K^T fragments), own-key K and V fragments -> registers
    {
      constexpr int PIECES = C::BN * C::CPR;
#pragma unroll
      for (int c = 0; c < PIECES / 256; ++c) {
        const int piece = tid + 256 * c;
        const int r = piece / C::CPR, col = piece % C::CPR;
        const int key = min(r, n_keys - 1);
        const u32x4 x = *reinterpret_cast<const u32x4*>(p.k + ((kv_row0 + key) * p.hkv + kvh) * D + col * 8);
        *reinterpret_cast<u32x4*>(smem + r * C::RSTRIDE + col * 16) = x;
      }
    }
    bf16x8 kf[D / 16], vf[D / 16];
    {
      const int64_t off = ((kv_row0 + my_key_ld) * p.hkv + kvh) * D + 8 * g2;
#pragma unroll
      for (int ks = 0; ks < D / 16; ++ks) {
        kf[ks] = *reinterpret_cast<const bf16x8*>(p.k + off + 16 * ks);
        vf[ks] = *reinterpret_cast<const bf16x8*>(p.v + off + 16 * ks);
      }
    }

    // ---- Q / dO block staging -------------------------------------------------------------
    u32x4 qreg[C::QPT], doreg[C::QPT];
    float statreg = 0.f;
    auto issue_loads = [&](int qb) {
#pragma unroll
      for (int c = 0; c < C::QPT; ++c) {
        const int piece = tid + 256 * c;
        const int r = piece / C::CPR, col = piece % C::CPR;
        const int row = min(qb * C::BM + r, w.q_len - 1);
        const int64_t off = ((int64_t)(w.q_local_off + row) * p.hq + head) * D + col * 8;
        qreg[c] = *reinterpret_cast<const u32x4*>(p.q + off);
        doreg[c] = *reinterpret_cast<const u32x4*>(p.d_o + off);
      }
      if (tid < 2 * C::BM) {
        const int r = tid & (C::BM - 1);
        const int row = min(qb * C::BM + r, w.q_len - 1);
        const int64_t off = (int64_t)head * p.tq + w.q_local_off + row;
        if (tid < C::BM) {
          const float l = p.lse[off];
          statreg = l == -INFINITY ? INFINITY : l * kLog2e;   // a row without keys contributes nothing
        } else {
          statreg = p.delta[off];
        }
      }
    };
    auto store_stage = [&](int buf) {
      unsigned char* qs = smem + C::OFF_STAGE + buf * C::STAGE;
      unsigned char* dos = qs + C::QBYTES;
#pragma unroll
      for (int c = 0; c < C::QPT; ++c) {
        const int piece = tid + 256 * c;
        const int r = piece / C::CPR, col = piece % C::CPR;
        *reinterpret_cast<u32x4*>(qs + r * C::RSTRIDE + col * 16) = qreg[c];
        *reinterpret_cast<u32x4*>(dos + r * C::RSTRIDE + col * 16) = doreg[c];
      }
      if (tid < 2 * C::BM) reinterpret_cast<float*>(dos + C::QBYTES)[tid] = statreg;
    };

    if (qb0 < qb1) {
      issue_loads(qb0);
      store_stage(0);
    }
    __syncthreads();

    // K^T fragments of this wave's channel slice for dQ = dS K: B operand, lane = channel
    // 32*wave + l32, k-slots = keys 16*ks + 8*g2 + [0,8)
    bf16x8 ktf[C::BN / 16];
    if (wave < D / 32) {
#pragma unroll
      for (int ks = 0; ks < C::BN / 16; ++ks) {
        const unsigned char* a0 = smem + (16 * ks + 8 * g2 + tr_row) * C::RSTRIDE + (32 * wave + tr_col) * 2;
        ktf[ks] = tr_read_8(a0, 4 * C::RSTRIDE);
      }
    }

    f32x16 dvacc[D / 32], dkacc[D / 32];
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
      for (int i = 0; i < 16; ++i) { dvacc[db][i] = 0.f; dkacc[db][i] = 0.f; }

    for (int qb = qb0; qb < qb1; ++qb) {
      const int buf = (qb - qb0) & 1;
      if (qb + 1 < qb1) issue_loads(qb + 1);
      const unsigned char* qs = smem + C::OFF_STAGE + buf * C::STAGE;
      const unsigned char* dos = qs + C::QBYTES;
      const float* stat = reinterpret_cast<const float*>(dos + C::QBYTES);
      unsigned char* dsm = smem + C::OFF_DS;

      const int row0 = qb * C::BM;
      const int q_pos0 = w.q_seq_start + row0;
      const int rows_here = min(C::BM, w.q_len - row0);
      // wave-uniform visibility of this wave's 32 keys from this query block
      const bool wave_sees = (32 * wave < n_keys) && (k_pos0 + 32 * wave <= q_pos0 + rows_here - 1);
      const bool need_mask = (k_pos0 + 32 * wave + 31 > q_pos0) || (32 * wave + 32 > n_keys) || (rows_here < C::BM);

      if (wave_sees) {
        // ---- S = Q K^T, dP = dO V^T   [32 rows x 32 own keys] -------------------------------
        f32x16 sacc, dpacc;
#pragma unroll
        for (int i = 0; i < 16; ++i) { sacc[i] = 0.f; dpacc[i] = 0.f; }
        const unsigned char* qrow = qs + l32 * C::RSTRIDE + 16 * g2;
        const unsigned char* dorow = dos + l32 * C::RSTRIDE + 16 * g2;
#pragma unroll
        for (int ks = 0; ks < D / 16; ++ks) {
          const bf16x8 aq = *reinterpret_cast<const bf16x8*>(qrow + 32 * ks);
          sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(aq, kf[ks], sacc, 0, 0, 0);
          const bf16x8 ado = *reinterpret_cast<const bf16x8*>(dorow + 32 * ks);
          dpacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ado, vf[ks], dpacc, 0, 0, 0);
        }
        // ---- P = exp2(s c - LSE2), dS = P (dP - delta); register i is row 8*(i/4) + 4*g2 + i%4
        bf16x8 pb[2], dsb[2];
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          const f32x4 lse4 = *reinterpret_cast<const f32x4*>(stat + 8 * r4 + 4 * g2);
          const f32x4 del4 = *reinterpret_cast<const f32x4*>(stat + C::BM + 8 * r4 + 4 * g2);
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int i = 4 * r4 + e;
            const int r = 8 * r4 + 4 * g2 + e;
            float pr = __builtin_amdgcn_exp2f(fmaf(sacc[i], p.scale_log2, -lse4[e]));
            if (need_mask && (!my_key_valid || r >= rows_here || my_k_pos > q_pos0 + r)) pr = 0.f;
            const float ds = pr * (dpacc[i] - del4[e]);
            pb[i / 8][i % 8] = (__bf16)pr;
            dsb[i / 8][i % 8] = (__bf16)ds;
            // dS to LDS as [row][key] for the dQ contraction
            *reinterpret_cast<__bf16*>(dsm + r * C::SSTRIDE + my_key * 2) = (__bf16)ds;
          }
        }
        // ---- dV^T += dO^T P,  dK^T += Q^T dS  [channel x own key] ----------------------------
        // k-slots of step t are rows 16t + 4*g2 + [0,4) and 16t + 8 + 4*g2 + [0,4), matching pb/dsb
#pragma unroll
        for (int t = 0; t < 2; ++t) {
#pragma unroll
          for (int db = 0; db < D / 32; ++db) {
            const int roff = (16 * t + 4 * g2 + tr_row) * C::RSTRIDE + (32 * db + tr_col) * 2;
            const bf16x8 a_do = tr_read_8(dos + roff, 8 * C::RSTRIDE);
            dvacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_do, pb[t], dvacc[db], 0, 0, 0);
            const bf16x8 a_q = tr_read_8(qs + roff, 8 * C::RSTRIDE);
            dkacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_q, dsb[t], dkacc[db], 0, 0, 0);
          }
        }
      } else {
        // keys of this wave are invisible to the block: their dS columns are zero
#pragma unroll
        for (int r = 0; r < 16; ++r)
          *reinterpret_cast<__bf16*>(dsm + (r + 16 * g2) * C::SSTRIDE + my_key * 2) = (__bf16)0.f;
      }
      __syncthreads();   // dS complete

      // ---- dQ slice: [32 rows x channels 32*wave..+31] = dS [32 x 128] K [128 x slice] -------
      if (wave < D / 32) {
        f32x16 dqacc;
#pragma unroll
        for (int i = 0; i < 16; ++i) dqacc[i] = 0.f;
        const unsigned char* dsrow = dsm + l32 * C::SSTRIDE + 16 * g2;
#pragma unroll
        for (int ks = 0; ks < C::BN / 16; ++ks) {
          const bf16x8 a = *reinterpret_cast<const bf16x8*>(dsrow + 32 * ks);
          dqacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, ktf[ks], dqacc, 0, 0, 0);
        }
        float* dqp = p.dq + ((int64_t)(w.q_local_off + row0) * p.hq + head) * D + 32 * wave + l32;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int r = 8 * (i / 4) + 4 * g2 + (i % 4);
          if (r < rows_here) unsafeAtomicAdd(dqp + (int64_t)r * p.hq * D, dqacc[i] * p.scale);
        }
      }
      if (qb + 1 < qb1) store_stage(buf ^ 1);
      __syncthreads();   // next stage visible; dS free for reuse
    }

    // ---- epilogue: dK^T, dV^T [channel x own key] -> pool accumulators -------------------------
    if (my_key_valid) {
      const int64_t off = ((kv_row0 + my_key) * p.hkv + kvh) * D;
#pragma unroll
      for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int c = 32 * db + 8 * (i / 4) + 4 * g2 + (i % 4);
          unsafeAtomicAdd(p.dv + off + c, dvacc[db][i]);
          unsafeAtomicAdd(p.dk + off + c, dkacc[db][i] * p.scale);
        }
    }
  }
}

}  // namespace
}  // namespace fcp

using fcp::fail;

extern "C" int fcp_attn_bwd_step(const void* q, const void* k, const void* v, const void* d_o, const float* lse,
                                 const float* delta, const int32_t* cu_seqlens_kv, int32_t n_seqs,
                                 const fcp_work_desc* work, int64_t n_work, int32_t tq, int32_t tkv, int32_t hq,
                                 int32_t hkv, int32_t head_dim, float softmax_scale, float* dq_acc, float* dk_acc,
                                 float* dv_acc, void* scratch, size_t scratch_bytes, void* stream) {
  fcp::clear_error();
  if (!q || !k || !v || !d_o || !lse || !delta || !cu_seqlens_kv || !dq_acc || !dk_acc || !dv_acc || !scratch)
    return fail(FCP_ERR_INVALID_ARG, "fcp_attn_bwd_step: null pointer");
  if (n_work > 0 && !work) return fail(FCP_ERR_INVALID_ARG, "fcp_attn_bwd_step: work is NULL");
  if (tq < 0 || tkv < 1 || n_seqs < 1 || n_work < 0 || hq < 1 || hkv < 1)
    return fail(FCP_ERR_INVALID_ARG, "fcp_attn_bwd_step: bad sizes");
  if (n_work > (1 << 24)) return fail(FCP_ERR_UNSUPPORTED, "fcp_attn_bwd_step: more than 2^24 work items");
  if (hq % hkv != 0) return fail(FCP_ERR_UNSUPPORTED, "fcp_attn_bwd_step: hq %d not a multiple of hkv %d", hq, hkv);
  if (head_dim != 64 && head_dim != 128) return fail(FCP_ERR_UNSUPPORTED, "fcp_attn_bwd_step: head_dim %d not 64/128", head_dim);
  if (!(softmax_scale > 0.f) || !(softmax_scale < 1e30f)) return fail(FCP_ERR_INVALID_ARG, "fcp_attn_bwd_step: softmax_scale must be positive and finite");
  const uintptr_t align_mask = reinterpret_cast<uintptr_t>(q) | reinterpret_cast<uintptr_t>(k) |
                               reinterpret_cast<uintptr_t>(v) | reinterpret_cast<uintptr_t>(d_o);
  if (align_mask & 15u) return fail(FCP_ERR_INVALID_ARG, "fcp_attn_bwd_step: q/k/v/d_o must be 16-byte aligned");
  if (reinterpret_cast<uintptr_t>(scratch) & 63u) return fail(FCP_ERR_INVALID_ARG, "fcp_attn_bwd_step: scratch must be 64-byte aligned");
  const size_t need = fcp_scratch_bytes(FCP_SCRATCH_BWD, tq, tkv, hq, hkv, head_dim, n_work, 1);
  if (scratch_bytes < need) return fail(FCP_ERR_CAPACITY, "fcp_attn_bwd_step: scratch %zu < %zu bytes", scratch_bytes, need);

  hipStream_t st = (hipStream_t)stream;
  const int64_t cap = fcp::bwd_tile_cap(tkv, n_work);
  if (cap > INT32_MAX / 64) return fail(FCP_ERR_UNSUPPORTED, "fcp_attn_bwd_step: too many tiles");
  int rc = fcp::launch_schedule(true, work, n_work, cu_seqlens_kv, n_seqs, tq, tkv, 1, cap, scratch, nullptr, 0, st);
  if (rc != FCP_OK) return rc;
  if (tq == 0 || n_work == 0) return FCP_OK;

  fcp::BwdParams p;
  p.q = (const uint16_t*)q; p.k = (const uint16_t*)k; p.v = (const uint16_t*)v; p.d_o = (const uint16_t*)d_o;
  p.lse = lse; p.delta = delta; p.cu = cu_seqlens_kv; p.work = work;
  p.hdr_ro = fcp::sched_header(scratch); p.hdr = (fcp::SchedHeader*)scratch;
  p.tiles = fcp::sched_tiles(scratch, n_work);
  p.dq = dq_acc; p.dk = dk_acc; p.dv = dv_acc;
  p.tq = tq; p.hq = hq; p.hkv = hkv;
  p.scale = softmax_scale; p.scale_log2 = softmax_scale * fcp::kLog2e;

  int dev = 0, n_cu = 256;
  FCP_HIP_CHECK(hipGetDevice(&dev));
  FCP_HIP_CHECK(hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev));
  int64_t units = cap * hq;
  int64_t blocks = (int64_t)n_cu;
  if (blocks > units) blocks = (units + 7) / 8 * 8;
  if (blocks < 8) blocks = 8;
  if (head_dim == 128) {
    static bool attr_done = false;
    if (!attr_done) {
      FCP_HIP_CHECK(hipFuncSetAttribute((const void*)fcp::bwd_kernel<128>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                        fcp::BwdCfg<128>::LDS_BYTES));
      attr_done = true;
    }
    hipLaunchKernelGGL(fcp::bwd_kernel<128>, dim3((unsigned)blocks), dim3(256), fcp::BwdCfg<128>::LDS_BYTES, st, p);
  } else {
    static bool attr_done = false;
    if (!attr_done) {
      FCP_HIP_CHECK(hipFuncSetAttribute((const void*)fcp::bwd_kernel<64>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                        fcp::BwdCfg<64>::LDS_BYTES));
      attr_done = true;
    }
    hipLaunchKernelGGL(fcp::bwd_kernel<64>, dim3((unsigned)blocks), dim3(256), fcp::BwdCfg<64>::LDS_BYTES, st, p);
  }
  FCP_HIP_CHECK(hipGetLastError());
  return FCP_OK;
}
