// fcp_attn_fwd_step: partial causal attention of one CP rank for its ring steps.
//
// Function computed: softmax(scale Q K^T) V (paper Eq. 1, Sec. 3.1) with the causal mask
// (Sec. 4.3), restricted to the keys one ring step brings (ring-style CP, Sec. 3.2), for
// packed sequences of heterogeneous length (Sec. 4.1).  Per row the kernel emits the
// locally normalised output and LSE = ln sum exp(scaled scores).
//
// gfx950 design
//   * persistent 256-thread blocks (4 wave64) pull (query tile, head) units from per-XCD
//     counters; the tile list is sorted longest-first by the scheduler kernel;
//   * a unit = 128 query rows of one work item for one query head; wave w owns rows
//     32w .. 32w+31 and keeps its Q fragments in registers for the whole unit;
//   * K/V stream through LDS in 64-key tiles, double buffered, global loads for tile t+1 in
//     flight while tile t is computed; one barrier per tile;
//   * scores are computed TRANSPOSED, S^T = K Q^T with v_mfma_f32_32x32x16_bf16: a lane then
//     holds 16 keys of ONE query column, so the row maximum and sum are in-lane reductions
//     plus a single exchange with the lane 32 away, and the exponentiated scores are already
//     in the B-operand layout of the second contraction O^T += V^T P^T;
//   * V^T fragments come from the row-major V tile through ds_read_b64_tr_b16 (LDS
//     transpose read), so V is never transposed in memory;
//   * key tiles that lie completely below the diagonal skip the mask; key tiles completely
//     above it are never visited (the loop bound comes from the last row's position).
#include "fcp_device.h"

namespace fcp {
namespace {

struct FwdParams {
  const uint16_t* q;
  const uint16_t* k;
  const uint16_t* v;
  SchedHeader* hdr;
  const Tile* tiles;
  float* o_part;
  float* lse_part;
  int32_t tq, hq, hkv;
  float scale_log2;  // softmax_scale * log2(e)
};

constexpr float kRescaleThreshold = 8.f;   // log2 units

template <int D>
struct FwdCfg {
  static constexpr int BM = kFwdBM;               // 128 query rows per unit (32 per wave)
  static constexpr int BN = kFwdBN;               // 64 keys per LDS tile
  static constexpr int KSTRIDE = D * 2 + 16;      // bytes; b128 row reads hit distinct banks
  static constexpr int VSTRIDE = D * 2 + 64;      // bytes; 4-row transpose reads hit distinct banks
  static constexpr int KBYTES = BN * KSTRIDE;
  static constexpr int VBYTES = BN * VSTRIDE;
  static constexpr int STAGE = KBYTES + VBYTES;
  static constexpr int LDS_BYTES = 2 * STAGE;
  static constexpr int CHUNKS = BN * D * 2 / 16;  // 16-byte pieces per tensor tile
  static constexpr int CPT = CHUNKS / 256;        // pieces per thread
  static constexpr int CPR = D * 2 / 16;          // pieces per row
  static constexpr int RPP = 256 / CPR;           // rows covered by one pass of the 256 threads
};

// On this chip plain VALU instructions do not overlap with MFMAs (measured: an MFMA plus n
// fp32 FMAs takes the sum of both), only the transcendental unit does.  The loop therefore
// spends as few VALU instructions per MFMA as it can: global loads go through buffer
// instructions whose per-tile offset is a scalar (out-of-range rows read as zero, so there is
// no clamping), LDS addresses are per-thread constants plus immediates, and the accumulator
// rescale is lazy.
template <int D>
__global__ __launch_bounds__(256, 2) void fwd_kernel(const FwdParams p) {
  using C = FwdCfg<D>;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  __shared__ int32_t s_next_unit;
  __shared__ int32_t s_rec[16];

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, g2 = lane >> 5;
  const int G = p.hq / p.hkv;

  // unit numbering: with hq % 8 == 0 each XCD owns a contiguous eighth of the heads
  const bool per_xcd = (p.hq % kNumXcd) == 0;
  const int xcd = per_xcd ? (int)(blockIdx.x % kNumXcd) : 0;
  const int heads_here = per_xcd ? p.hq / kNumXcd : p.hq;
  UnitQueue uq;
  uq.init(p.hdr, p.tiles, xcd, heads_here, &s_next_unit, s_rec);

  // per-thread constants of the K/V tile movement
  const int ld_r = tid / C::CPR, ld_c = tid % C::CPR;
  const int lds_k_thread = ld_r * C::KSTRIDE + ld_c * 16;
  const int lds_v_thread = C::KBYTES + ld_r * C::VSTRIDE + ld_c * 16;
  const int kv_row_bytes = p.hkv * D * 2;
  const int voff0 = ld_r * kv_row_bytes + ld_c * 16;

  for (;;) {
    const int unit = uq.current(&s_next_unit);
    if (unit >= uq.n_units) break;
    const QTile t = read_record<QTile>(s_rec);
    const int head = xcd * heads_here + unit % heads_here;
    const int kvh = head / G;
    uq.prefetch();   // next unit's record and the following unit's number start their trips now

    const int wave_r0 = wave * 32;
    const bool wave_active = wave_r0 < t.rows;
    const int my_row = wave_r0 + l32;
    const bool row_valid = my_row < t.rows;
    const int row_ld = min(my_row, t.rows - 1);
    const int q_pos = t.q_pos0 + my_row;
    const int wave_first_pos = t.q_pos0 + wave_r0;
    const int wave_last_pos = t.q_pos0 + min(wave_r0 + 31, t.rows - 1);

    // Q fragments: B operand of S^T = K Q^T.  Lane holds column q = l32, channels 16*ks + 8*g2 + [0,8)
    bf16x8 qf[D / 16];
    {
      const uint16_t* qp = p.q + ((int64_t)(t.q_row0 + row_ld) * p.hq + head) * D + 8 * g2;
#pragma unroll
      for (int ks = 0; ks < D / 16; ++ks) qf[ks] = *reinterpret_cast<const bf16x8*>(qp + 16 * ks);
    }

    // Key segments: a buffer resource per segment whose extent ends with the last visible key,
    // so rows past it load as zeros.
    const int nt0 = (t.vis[0] + C::BN - 1) / C::BN, nt1 = (t.vis[1] + C::BN - 1) / C::BN;
    const int n_iter = nt0 + nt1;
    __amdgpu_buffer_rsrc_t rk[2], rv[2];
#pragma unroll
    for (int s = 0; s < 2; ++s) {
      const int64_t off = ((int64_t)t.kv_row0[s] * p.hkv + kvh) * D;
      const int bytes = t.vis[s] > 0 ? (t.vis[s] - 1) * kv_row_bytes + D * 2 : 0;
      rk[s] = __builtin_amdgcn_make_buffer_rsrc((void*)(p.k + off), (short)0, bytes, 0x00020000);
      rv[s] = __builtin_amdgcn_make_buffer_rsrc((void*)(p.v + off), (short)0, bytes, 0x00020000);
    }

    f32x16 oacc[D / 32];
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
      for (int i = 0; i < 16; ++i) oacc[db][i] = 0.f;
    float m_run = -INFINITY;   // running maximum in log2 units (score * scale_log2)
    float l_run = 0.f;         // this lane's share of the running sum

    // ---- K/V tile movement ---------------------------------------------------------
    u32x4 kreg[C::CPT], vreg[C::CPT];
    auto issue_loads = [&](int it) {
      const int s = it >= nt0 ? 1 : 0;
      const int soff = (it - (s ? nt0 : 0)) * (C::BN * kv_row_bytes);
#pragma unroll
      for (int c = 0; c < C::CPT; ++c) {
        const int voff = voff0 + c * C::RPP * kv_row_bytes;
        if (s == 0) {
          kreg[c] = __builtin_amdgcn_raw_buffer_load_b128(rk[0], voff, soff, 0);
          vreg[c] = __builtin_amdgcn_raw_buffer_load_b128(rv[0], voff, soff, 0);
        } else {
          kreg[c] = __builtin_amdgcn_raw_buffer_load_b128(rk[1], voff, soff, 0);
          vreg[c] = __builtin_amdgcn_raw_buffer_load_b128(rv[1], voff, soff, 0);
        }
      }
    };
    auto store_tile = [&](int buf) {
      unsigned char* kb = smem + buf * C::STAGE + lds_k_thread;
      unsigned char* vb = smem + buf * C::STAGE + lds_v_thread;
#pragma unroll
      for (int c = 0; c < C::CPT; ++c) {
        *reinterpret_cast<u32x4*>(kb + c * C::RPP * C::KSTRIDE) = kreg[c];
        *reinterpret_cast<u32x4*>(vb + c * C::RPP * C::VSTRIDE) = vreg[c];
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

      const int s = it >= nt0 ? 1 : 0;
      const int kt = it - (s ? nt0 : 0);
      const int k_pos0 = t.k_pos0[s] + kt * C::BN;            // position of the tile's first key
      const int n_valid = min(C::BN, t.vis[s] - kt * C::BN);   // keys of the tile inside the segment
      // wave-uniform: does this wave see anything in the tile / need the element mask?
      const bool wave_sees = wave_active && k_pos0 <= wave_last_pos;
      const bool need_mask = (k_pos0 + C::BN - 1 > wave_first_pos) || (n_valid < C::BN);

      if (wave_sees) {
        const unsigned char* kb = smem + buf * C::STAGE;
        const unsigned char* vb = kb + C::KBYTES;
        // LDS fragments are requested a whole group ahead of the MFMAs that use them (the
        // sched_barriers keep the compiler from re-serialising read -> wait -> MFMA).
        // A operand of O^T += V^T P^T: rows d = 32*db + l32; its 8 k-slots are keys
        // 16t + {4*g2 + [0,4), 8 + 4*g2 + [0,4)}.  Transpose read: a lane supplies the address of row
        // (l%16)/4, channels 4*(l%4) + [0,4) of its 16-lane block; block b covers channels
        // 16*(b%2) + [0,16) for key group g2 = b/2.
        const unsigned char* vbase = vb + (4 * g2 + ((lane & 15) >> 2)) * C::VSTRIDE +
                                     (16 * ((lane >> 4) & 1) + 4 * (lane & 3)) * 2;
        auto load_vt = [&](int tt, bf16x8 (&dst)[D / 32]) {
#pragma unroll
          for (int db = 0; db < D / 32; ++db) {
            const unsigned char* a0 = vbase + (16 * tt) * C::VSTRIDE + 64 * db;
            const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                (__attribute__((address_space(3))) s16x4*)(a0));
            const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                (__attribute__((address_space(3))) s16x4*)(a0 + 8 * C::VSTRIDE));
            dst[db] = __builtin_shufflevector(__builtin_bit_cast(bf16x4, lo), __builtin_bit_cast(bf16x4, hi),
                                              0, 1, 2, 3, 4, 5, 6, 7);
          }
        };
        // ---- S^T[key, q] = K Q^T ------------------------------------------------------
        f32x16 sacc[2];
        bf16x8 ka[2][D / 16];
        const unsigned char* krow = kb + l32 * C::KSTRIDE + 16 * g2;
#pragma unroll
        for (int ks = 0; ks < D / 16; ++ks) ka[0][ks] = *reinterpret_cast<const bf16x8*>(krow + 32 * ks);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int ks = 0; ks < D / 16; ++ks)
          ka[1][ks] = *reinterpret_cast<const bf16x8*>(krow + 32 * C::KSTRIDE + 32 * ks);
        {
          const f32x16 z = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
          sacc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[0][0], qf[0], z, 0, 0, 0);
#pragma unroll
          for (int ks = 1; ks < D / 16; ++ks)
            sacc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[0][ks], qf[ks], sacc[0], 0, 0, 0);
          __builtin_amdgcn_sched_barrier(0);
          sacc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[1][0], qf[0], z, 0, 0, 0);
#pragma unroll
          for (int ks = 1; ks < D / 16; ++ks)
            sacc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[1][ks], qf[ks], sacc[1], 0, 0, 0);
        }
        bf16x8 vt0[D / 32], vt1[D / 32];
        load_vt(0, vt0);     // lands while the scores are exponentiated
        load_vt(1, vt1);
        __builtin_amdgcn_sched_barrier(0);
        // ---- mask + online softmax ------------------------------------------------------
        // register i of block kbk is key 32*kbk + 8*(i/4) + 4*g2 + (i%4) of the tile
        if (need_mask) {
#pragma unroll
          for (int kbk = 0; kbk < 2; ++kbk)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
              const int kk = 32 * kbk + 8 * (i / 4) + 4 * g2 + (i % 4);
              if (kk >= n_valid || k_pos0 + kk > q_pos) sacc[kbk][i] = -INFINITY;
            }
        }
        float mx = -INFINITY;
#pragma unroll
        for (int kbk = 0; kbk < 2; ++kbk)
#pragma unroll
          for (int i = 0; i < 16; ++i) mx = fmaxf(mx, sacc[kbk][i]);
        mx = lane32_partner_max(mx) * p.scale_log2;
        // Lazy rescale: the running maximum is raised only when some row of the wave outgrows it by
        // 2^kRescaleThreshold; until then probabilities may exceed 1 (by at most that factor).
        if (__builtin_amdgcn_ballot_w64(mx > m_run + kRescaleThreshold) != 0) {
          const float m_new = fmaxf(m_run, mx);
          const float alpha = __builtin_amdgcn_exp2f(m_run - (m_new == -INFINITY ? 0.f : m_new));
          m_run = m_new;
          l_run *= alpha;
#pragma unroll
          for (int db = 0; db < D / 32; ++db)
#pragma unroll
            for (int i = 0; i < 16; ++i) oacc[db][i] *= alpha;
        }
        const float m_use = m_run == -INFINITY ? 0.f : m_run;
        float psum = 0.f;
        bf16x8 pf[4];   // P^T as B operand: k-step t covers keys 16t..16t+15 of the tile
        // the row sum is taken over the unrounded fp32 values: summing the bf16-rounded ones
        // (v_dot2c) would halve the adds but costs up to 2^-9 relative on a peaked row, i.e.
        // more than the 1e-3 the LSE has to hold
#pragma unroll
        for (int kbk = 0; kbk < 2; ++kbk)
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            const float e = __builtin_amdgcn_exp2f(fmaf(sacc[kbk][i], p.scale_log2, -m_use));
            psum += e;
            pf[2 * kbk + i / 8][i % 8] = (__bf16)e;
          }
        l_run += psum;
        __builtin_amdgcn_sched_barrier(0);
        // ---- O^T[d, q] += V^T P^T ---------------------------------------------------------
        bf16x8 vt2[D / 32], vt3[D / 32];
        load_vt(2, vt2);
        load_vt(3, vt3);
#pragma unroll
        for (int db = 0; db < D / 32; ++db) oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vt0[db], pf[0], oacc[db], 0, 0, 0);
#pragma unroll
        for (int db = 0; db < D / 32; ++db) oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vt1[db], pf[1], oacc[db], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int db = 0; db < D / 32; ++db) oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vt2[db], pf[2], oacc[db], 0, 0, 0);
#pragma unroll
        for (int db = 0; db < D / 32; ++db) oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vt3[db], pf[3], oacc[db], 0, 0, 0);
      }

      if (it + 1 < n_iter) store_tile(buf ^ 1);
      __syncthreads();
    }

    // ---- epilogue: normalise, write partial O (fp32) and LSE --------------------------------
    const float l_tot = lane32_partner_sum(l_run);
    const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
    if (row_valid) {
      float* orow = p.o_part + (int64_t)t.step * ((int64_t)p.tq * p.hq * D) +
                    ((int64_t)(t.q_row0 + my_row) * p.hq + head) * D;
#pragma unroll
      for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          f32x4 o4 = {oacc[db][4 * r4] * inv, oacc[db][4 * r4 + 1] * inv, oacc[db][4 * r4 + 2] * inv,
                      oacc[db][4 * r4 + 3] * inv};
          *reinterpret_cast<f32x4*>(orow + 32 * db + 8 * r4 + 4 * g2) = o4;
        }
      if (g2 == 0) {
        const float lse = l_tot > 0.f ? (m_run + __builtin_amdgcn_logf(l_tot)) * kLn2 : -INFINITY;
        p.lse_part[(int64_t)t.step * ((int64_t)p.hq * p.tq) + (int64_t)head * p.tq + t.q_row0 + my_row] = lse;
      }
    }
    uq.advance(&s_next_unit, s_rec);   // hand the next unit to the block
  }
}

}  // namespace
}  // namespace fcp

using fcp::fail;

extern "C" int fcp_attn_fwd_step(const void* q, const void* k, const void* v, const int32_t* cu_seqlens_kv,
                                 int32_t n_seqs, const fcp_work_desc* work, int64_t n_work, int32_t n_parts,
                                 int32_t tq, int32_t tkv, int32_t hq, int32_t hkv, int32_t head_dim,
                                 float softmax_scale, float* o_part, float* lse_part, void* scratch,
                                 size_t scratch_bytes, void* stream) {
  fcp::clear_error();
  if (!q || !k || !v || !cu_seqlens_kv || !o_part || !lse_part || !scratch)
    return fail(FCP_ERR_INVALID_ARG, "fcp_attn_fwd_step: null pointer");
  if (n_work > 0 && !work) return fail(FCP_ERR_INVALID_ARG, "fcp_attn_fwd_step: work is NULL");
  if (tq < 0 || tkv < 1 || n_seqs < 1 || n_work < 0 || n_parts < 1 || hq < 1 || hkv < 1)
    return fail(FCP_ERR_INVALID_ARG, "fcp_attn_fwd_step: bad sizes");
  if (n_work > (1 << 24)) return fail(FCP_ERR_UNSUPPORTED, "fcp_attn_fwd_step: more than 2^24 work items");
  if (hq % hkv != 0) return fail(FCP_ERR_UNSUPPORTED, "fcp_attn_fwd_step: hq %d not a multiple of hkv %d", hq, hkv);
  if (head_dim != 64 && head_dim != 128) return fail(FCP_ERR_UNSUPPORTED, "fcp_attn_fwd_step: head_dim %d not 64/128", head_dim);
  if (!(softmax_scale > 0.f) || !(softmax_scale < 1e30f)) return fail(FCP_ERR_INVALID_ARG, "fcp_attn_fwd_step: softmax_scale must be positive and finite");
  const uintptr_t align_mask = reinterpret_cast<uintptr_t>(q) | reinterpret_cast<uintptr_t>(k) |
                               reinterpret_cast<uintptr_t>(v) | reinterpret_cast<uintptr_t>(o_part);
  if (align_mask & 15u) return fail(FCP_ERR_INVALID_ARG, "fcp_attn_fwd_step: q/k/v/o_part must be 16-byte aligned");
  if (reinterpret_cast<uintptr_t>(scratch) & 63u) return fail(FCP_ERR_INVALID_ARG, "fcp_attn_fwd_step: scratch must be 64-byte aligned");
  const size_t need = fcp_scratch_bytes(FCP_SCRATCH_FWD, tq, tkv, hq, hkv, head_dim, n_work, n_parts);
  if (scratch_bytes < need) return fail(FCP_ERR_CAPACITY, "fcp_attn_fwd_step: scratch %zu < %zu bytes", scratch_bytes, need);
  if ((int64_t)tq * hq * head_dim * (int64_t)n_parts > ((int64_t)1 << 40))
    return fail(FCP_ERR_UNSUPPORTED, "fcp_attn_fwd_step: partial output too large");

  hipStream_t st = (hipStream_t)stream;
  const int64_t cap = fcp::q_tile_cap(tq, tkv, n_work, n_parts);
  if (cap > INT32_MAX / 64) return fail(FCP_ERR_UNSUPPORTED, "fcp_attn_fwd_step: too many tiles");
  int rc = fcp::launch_schedule(false, fcp::kFwdBM, fcp::kFwdBN, (int64_t)hkv * head_dim * 2, work, n_work, cu_seqlens_kv, n_seqs, tq, tkv, n_parts, cap, scratch,
                                lse_part, (int64_t)n_parts * hq * tq, st);
  if (rc != FCP_OK) return rc;
  if (tq == 0 || n_work == 0) return FCP_OK;

  fcp::FwdParams p;
  p.q = (const uint16_t*)q; p.k = (const uint16_t*)k; p.v = (const uint16_t*)v;
  p.hdr = (fcp::SchedHeader*)scratch;
  p.tiles = fcp::sched_tiles(scratch, n_work);
  p.o_part = o_part; p.lse_part = lse_part;
  p.tq = tq; p.hq = hq; p.hkv = hkv;
  p.scale_log2 = softmax_scale * 1.4426950408889634f;

  int dev = 0, n_cu = 256;
  FCP_HIP_CHECK(hipGetDevice(&dev));
  FCP_HIP_CHECK(hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev));
  int64_t units = cap * hq;
  int64_t blocks = (int64_t)n_cu * 2;
  if (blocks > units) blocks = (units + 7) / 8 * 8;   // keep a multiple of the XCD count
  if (blocks < 8) blocks = 8;
  if (head_dim == 128) {
    static bool attr_done = false;
    if (!attr_done) {
      FCP_HIP_CHECK(hipFuncSetAttribute((const void*)fcp::fwd_kernel<128>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                        fcp::FwdCfg<128>::LDS_BYTES));
      attr_done = true;
    }
    hipLaunchKernelGGL(fcp::fwd_kernel<128>, dim3((unsigned)blocks), dim3(256), fcp::FwdCfg<128>::LDS_BYTES, st, p);
  } else {
    static bool attr_done = false;
    if (!attr_done) {
      FCP_HIP_CHECK(hipFuncSetAttribute((const void*)fcp::fwd_kernel<64>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                        fcp::FwdCfg<64>::LDS_BYTES));
      attr_done = true;
    }
    hipLaunchKernelGGL(fcp::fwd_kernel<64>, dim3((unsigned)blocks), dim3(256), fcp::FwdCfg<64>::LDS_BYTES, st, p);
  }
  FCP_HIP_CHECK(hipGetLastError());
  return FCP_OK;
}
