// fcp_attn_bwd_step: gradient contributions of one CP rank for its ring steps.
//
// Backward of O = softmax(scale Q K^T) V (paper Eq. 1, Sec. 3.1; causal mask, Sec. 4.3) for
// the key sets the ring steps bring (ring-style CP, Sec. 3.2).  With the merged LSE the
// probabilities of a step are recomputed exactly, P = exp(scale s - LSE), so each step adds
// its own share:  dV += P^T dO,  dS = P o (dO V^T - delta),  dQ += scale dS K,  dK += scale dS^T Q.
//
// gfx950 design: two persistent kernels, because fp32 atomics retire at about one element
// per L2 channel per clock on this chip (~270 G/s), far too few to accumulate dQ per key tile.
//
//   dkv_kernel  unit = 128 keys of one segment of one work item x one KV head.  Wave w owns keys
//               32w..32w+31: their K and V fragments and the fp32 accumulators dK^T, dV^T
//               [channel x key] stay in registers while the unit loops over the query heads of
//               the KV head and over the 32-row query blocks that see the tile.  S = Q K^T and
//               dP = dO V^T come out as [query x key] with the key on the lane, which is exactly
//               the B-operand layout of dV^T += dO^T P and dK^T += Q^T dS; dO^T / Q^T are
//               transpose reads of the row-major LDS tiles.
//   dq_kernel   unit = 128 query rows of one work item x one query head (the forward's shape).
//               Wave w owns 32 rows, keeps Q and dO fragments in registers, streams K/V tiles
//               through LDS, forms S^T = K Q^T and dP^T = V dO^T [key x query] so that dS^T is
//               the B operand of dQ^T += K^T dS^T with K^T from transpose reads.
//
// Both add their result to the caller's fp32 accumulators once per unit: with plain
// load-add-store when the scheduler found that no other item of the launch touches the same
// rows (always the case for degree-1 sequences), otherwise with fp32 atomics.
#include "fcp_bwd.h"

namespace fcp {
namespace {

// ============================================================================================
// dQ
// ============================================================================================
template <int D>
struct DqCfg {
  static constexpr int BM = kDqBM;                // 128 query rows per unit (32 per wave)
  static constexpr int BN = kDqBN;                // 64 keys per LDS tile
  static constexpr int KSTRIDE = D * 2 + 32;      // K rows: b128 row reads AND transpose reads
  static constexpr int VSTRIDE = D * 2 + 16;      // V rows: b128 row reads only
  static constexpr int KBYTES = BN * KSTRIDE;
  static constexpr int VBYTES = BN * VSTRIDE;
  static constexpr int STAGE = KBYTES + VBYTES;
  static constexpr int LDS_BYTES = 2 * STAGE;
  static constexpr int CHUNKS = BN * D * 2 / 16;
  static constexpr int CPT = CHUNKS / 256;
  static constexpr int CPR = D * 2 / 16;
};

template <int D>
__global__ __launch_bounds__(256, 2) void dq_kernel(const BwdParams p) {
  using C = DqCfg<D>;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  __shared__ int32_t s_unit;

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, g2 = lane >> 5;
  const int G = p.hq / p.hkv;
  const bool per_xcd = (p.hq % kNumXcd) == 0;
  const int xcd = per_xcd ? (int)(blockIdx.x % kNumXcd) : 0;
  const int heads_here = per_xcd ? p.hq / kNumXcd : p.hq;
  const int n_units = p.hdr->n_tiles * heads_here;

  for (;;) {
    if (tid == 0) s_unit = atomicAdd(&p.hdr->counter[xcd], 1);
    __syncthreads();
    const int unit = __builtin_amdgcn_readfirstlane(s_unit);
    __syncthreads();
    if (unit >= n_units) break;
    const int tile_i = unit / heads_here;
    const int head = xcd * heads_here + unit % heads_here;
    const int kvh = head / G;
    const QTile t = *reinterpret_cast<const QTile*>(&p.tiles[tile_i]);
    const bool exclusive = (t.flags & kFlagQExclusive) != 0;

    const int rows_here = t.rows;
    const int wave_r0 = wave * 32;
    const bool wave_active = wave_r0 < rows_here;
    const int my_row = wave_r0 + l32;
    const bool row_valid = my_row < rows_here;
    const int row_ld = min(my_row, rows_here - 1);
    const int q_pos = t.q_pos0 + my_row;
    const int wave_first_pos = t.q_pos0 + wave_r0;
    const int wave_last_pos = t.q_pos0 + min(wave_r0 + 31, rows_here - 1);

    // Q and dO fragments: B operands (lane = query column), channels 16*ks + 8*g2 + [0,8)
    bf16x8 qf[D / 16], dof[D / 16];
    {
      const int64_t off = ((int64_t)(t.q_row0 + row_ld) * p.hq + head) * D + 8 * g2;
#pragma unroll
      for (int ks = 0; ks < D / 16; ++ks) {
        qf[ks] = *reinterpret_cast<const bf16x8*>(p.q + off + 16 * ks);
        dof[ks] = *reinterpret_cast<const bf16x8*>(p.d_o + off + 16 * ks);
      }
    }
    float lse2, delta;
    {
      const int64_t off = (int64_t)head * p.tq + t.q_row0 + row_ld;
      const float l = p.lse[off];
      lse2 = l == -INFINITY ? INFINITY : l * kLog2e;
      delta = p.delta[off];
    }

    int vis[2], nt[2], k_seg_pos[2];
    int64_t kv_row0[2];
#pragma unroll
    for (int s = 0; s < 2; ++s) {
      vis[s] = t.vis[s];
      nt[s] = (vis[s] + C::BN - 1) / C::BN;
      kv_row0[s] = t.kv_row0[s];
      k_seg_pos[s] = t.k_pos0[s];
    }
    const int n_iter = nt[0] + nt[1];

    f32x16 dqacc[D / 32];
#pragma unroll
    for (int db = 0; db < D / 32; ++db) dqacc[db] = zero16();

    u32x4 kreg[C::CPT], vreg[C::CPT];
    auto issue_loads = [&](int it) {
      const int s = it >= nt[0] ? 1 : 0;
      const int kt = it - (s ? nt[0] : 0);
      const int vl = vis[s];
#pragma unroll
      for (int c = 0; c < C::CPT; ++c) {
        const int piece = tid + 256 * c;
        const int r = piece / C::CPR, col = piece % C::CPR;
        const int key = min(kt * C::BN + r, vl - 1);
        const int64_t off = ((kv_row0[s] + key) * p.hkv + kvh) * D + col * 8;
        kreg[c] = *reinterpret_cast<const u32x4*>(p.k + off);
        vreg[c] = *reinterpret_cast<const u32x4*>(p.v + off);
      }
    };
    auto store_tile = [&](int buf) {
      unsigned char* kb = smem + buf * C::STAGE;
      unsigned char* vb = kb + C::KBYTES;
#pragma unroll
      for (int c = 0; c < C::CPT; ++c) {
        const int piece = tid + 256 * c;
        const int r = piece / C::CPR, col = piece % C::CPR;
        *reinterpret_cast<u32x4*>(kb + r * C::KSTRIDE + col * 16) = kreg[c];
        *reinterpret_cast<u32x4*>(vb + r * C::VSTRIDE + col * 16) = vreg[c];
      }
    };

    if (n_iter > 0) {
      issue_loads(0);
      store_tile(0);
    }
    __syncthreads();

    for (int it = 0; it < n_iter; ++it) {
      const int buf = it & 1;
      if (it + 1 < n_iter) issue_loads(it + 1);
      const int s = it >= nt[0] ? 1 : 0;
      const int kt = it - (s ? nt[0] : 0);
      const int k_pos0 = k_seg_pos[s] + kt * C::BN;
      const int n_valid = min(C::BN, vis[s] - kt * C::BN);
      const bool wave_sees = wave_active && k_pos0 <= wave_last_pos;
      const bool need_mask = (k_pos0 + C::BN - 1 > wave_first_pos) || (n_valid < C::BN);

      if (wave_sees) {
        const unsigned char* kb = smem + buf * C::STAGE;
        const unsigned char* vb = kb + C::KBYTES;
        // S^T = K Q^T and dP^T = V dO^T   [key x query], two 32-key blocks
        f32x16 sacc[2], dpacc[2];
#pragma unroll
        for (int kbk = 0; kbk < 2; ++kbk) {
          sacc[kbk] = zero16();
          dpacc[kbk] = zero16();
          const unsigned char* krow = kb + (32 * kbk + l32) * C::KSTRIDE + 16 * g2;
          const unsigned char* vrow = vb + (32 * kbk + l32) * C::VSTRIDE + 16 * g2;
#pragma unroll
          for (int ks = 0; ks < D / 16; ++ks) {
            const bf16x8 ak = *reinterpret_cast<const bf16x8*>(krow + 32 * ks);
            sacc[kbk] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ak, qf[ks], sacc[kbk], 0, 0, 0);
            const bf16x8 av = *reinterpret_cast<const bf16x8*>(vrow + 32 * ks);
            dpacc[kbk] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, dof[ks], dpacc[kbk], 0, 0, 0);
          }
        }
        // dS^T = P^T o (dP^T - delta); register i of block kbk is key 32*kbk + 8*(i/4) + 4*g2 + i%4
        bf16x8 dsf[4];
#pragma unroll
        for (int kbk = 0; kbk < 2; ++kbk)
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            float pr = __builtin_amdgcn_exp2f(fmaf(sacc[kbk][i], p.scale_log2, -lse2));
            if (need_mask) {
              const int kk = 32 * kbk + 8 * (i / 4) + 4 * g2 + (i % 4);
              if (kk >= n_valid || k_pos0 + kk > q_pos) pr = 0.f;
            }
            dsf[2 * kbk + i / 8][i % 8] = (__bf16)(pr * (dpacc[kbk][i] - delta));
          }
        // dQ^T[channel, query] += K^T dS^T; A operand by transpose reads of the K tile
        const unsigned char* kbase = kb + (4 * g2 + ((lane & 15) >> 2)) * C::KSTRIDE +
                                     (16 * ((lane >> 4) & 1) + 4 * (lane & 3)) * 2;
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
          for (int db = 0; db < D / 32; ++db) {
            const bf16x8 a = tr_read_8(kbase + (16 * t) * C::KSTRIDE + 64 * db, 8 * C::KSTRIDE);
            dqacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, dsf[t], dqacc[db], 0, 0, 0);
          }
      }
      if (it + 1 < n_iter) store_tile(buf ^ 1);
      __syncthreads();
    }

    // epilogue: dQ^T [channel x query] * scale -> accumulator rows
    if (row_valid) {
      float* dqp = p.dq + ((int64_t)(t.q_row0 + my_row) * p.hq + head) * D + 4 * g2;
#pragma unroll
      for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          const int c = 32 * db + 8 * r4;
          if (exclusive) {
            f32x4 a = *reinterpret_cast<f32x4*>(dqp + c);
#pragma unroll
            for (int e = 0; e < 4; ++e) a[e] += dqacc[db][4 * r4 + e] * p.scale;
            *reinterpret_cast<f32x4*>(dqp + c) = a;
          } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) unsafeAtomicAdd(dqp + c + e, dqacc[db][4 * r4 + e] * p.scale);
          }
        }
    }
  }
}

template <typename K>
int set_lds_once(K kernel, int bytes, bool* done) {
  if (!*done) {
    FCP_HIP_CHECK(hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes));
    *done = true;
  }
  return FCP_OK;
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
                               reinterpret_cast<uintptr_t>(v) | reinterpret_cast<uintptr_t>(d_o) |
                               reinterpret_cast<uintptr_t>(dq_acc) | reinterpret_cast<uintptr_t>(dk_acc) |
                               reinterpret_cast<uintptr_t>(dv_acc);
  if (align_mask & 15u) return fail(FCP_ERR_INVALID_ARG, "fcp_attn_bwd_step: tensors must be 16-byte aligned");
  if (reinterpret_cast<uintptr_t>(scratch) & 255u) return fail(FCP_ERR_INVALID_ARG, "fcp_attn_bwd_step: scratch must be 256-byte aligned");
  const size_t need = fcp_scratch_bytes(FCP_SCRATCH_BWD, tq, tkv, hq, hkv, head_dim, n_work, 1);
  if (scratch_bytes < need) return fail(FCP_ERR_CAPACITY, "fcp_attn_bwd_step: scratch %zu < %zu bytes", scratch_bytes, need);

  if ((int64_t)tq * hq * head_dim * 2 >= ((int64_t)1 << 31))
    return fail(FCP_ERR_UNSUPPORTED, "fcp_attn_bwd_step: tq * hq * head_dim * 2 must stay below 2^31 bytes");
  hipStream_t st = (hipStream_t)stream;
  const int64_t cap_kv = fcp::kv_tile_cap(tkv, n_work);
  const int64_t cap_q = fcp::q_tile_cap(tq, tkv, n_work, 1 << 20);
  if (cap_kv > INT32_MAX / 64 || cap_q > INT32_MAX / 64) return fail(FCP_ERR_UNSUPPORTED, "fcp_attn_bwd_step: too many tiles");
  void* region_kv = scratch;
  void* region_q = static_cast<char*>(scratch) + fcp::sched_region_bytes(n_work, cap_kv);
  float* stats = reinterpret_cast<float*>(static_cast<char*>(region_q) + fcp::sched_region_bytes(n_work, cap_q));
  int rc = fcp::launch_schedule(true, fcp::kBwdBN, fcp::kBwdBM, (int64_t)hkv * head_dim * 2, work, n_work, cu_seqlens_kv, n_seqs, tq, tkv, 1, cap_kv, region_kv, nullptr, 0, st);
  if (rc != FCP_OK) return rc;
  rc = fcp::launch_schedule(false, fcp::kDqBM, fcp::kDqBN, (int64_t)hkv * head_dim * 2, work, n_work, cu_seqlens_kv, n_seqs, tq, tkv, 1, cap_q, region_q, nullptr, 0, st);
  if (rc != FCP_OK) return rc;
  if (tq == 0 || n_work == 0) return FCP_OK;
  if ((rc = fcp::launch_row_stats(lse, delta, (int64_t)hq * tq, stats, st)) != FCP_OK) return rc;

  fcp::BwdParams p;
  p.q = (const uint16_t*)q; p.k = (const uint16_t*)k; p.v = (const uint16_t*)v; p.d_o = (const uint16_t*)d_o;
  p.lse = lse; p.delta = delta; p.stats = stats;
  p.dq = dq_acc; p.dk = dk_acc; p.dv = dv_acc;
  p.tq = tq; p.hq = hq; p.hkv = hkv;
  p.scale = softmax_scale; p.scale_log2 = softmax_scale * fcp::kLog2e;

  int dev = 0, n_cu = 256;
  FCP_HIP_CHECK(hipGetDevice(&dev));
  FCP_HIP_CHECK(hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev));
  auto grid_for = [&](int64_t units, int per_cu) {
    int64_t blocks = (int64_t)n_cu * per_cu;
    if (blocks > units) blocks = (units + 7) / 8 * 8;   // a multiple of the XCD count
    if (blocks < 8) blocks = 8;
    return dim3((unsigned)blocks);
  };

  // dK/dV over key tiles
  p.hdr = (fcp::SchedHeader*)region_kv;
  p.tiles = fcp::sched_tiles(region_kv, n_work);
  if ((rc = fcp::launch_dkv(p, head_dim, cap_kv * hkv, n_cu, st)) != FCP_OK) return rc;

  // dQ over query tiles
  p.hdr = (fcp::SchedHeader*)region_q;
  p.tiles = fcp::sched_tiles(region_q, n_work);
  if (head_dim == 128) {
    static bool done = false;
    if ((rc = fcp::set_lds_once(fcp::dq_kernel<128>, fcp::DqCfg<128>::LDS_BYTES, &done)) != FCP_OK) return rc;
    hipLaunchKernelGGL(fcp::dq_kernel<128>, grid_for(cap_q * hq, 2), dim3(256), fcp::DqCfg<128>::LDS_BYTES, st, p);
  } else {
    static bool done = false;
    if ((rc = fcp::set_lds_once(fcp::dq_kernel<64>, fcp::DqCfg<64>::LDS_BYTES, &done)) != FCP_OK) return rc;
    hipLaunchKernelGGL(fcp::dq_kernel<64>, grid_for(cap_q * hq, 2), dim3(256), fcp::DqCfg<64>::LDS_BYTES, st, p);
  }
  FCP_HIP_CHECK(hipGetLastError());
  return FCP_OK;
}
