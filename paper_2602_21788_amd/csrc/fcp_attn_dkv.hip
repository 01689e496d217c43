// dK / dV part of fcp_attn_bwd_step.
//
// Backward of O = softmax(scale Q K^T) V (paper Eq. 1, Sec. 3.1; causal mask, Sec. 4.3) for the key sets the
// ring steps bring (ring-style CP, Sec. 3.2).  With the merged LSE the probabilities of a step are recomputed
// exactly, P = exp(scale s - LSE), so each step adds its own share:
//   dV += P^T dO,   dS = P o (dO V^T - delta),   dK += scale dS^T Q,
// summed over the query heads of a KV head and over the query rows that see the key.
//
// gfx950 design
//   * persistent 1024-thread blocks (16 wave64, one block per CU, four waves per SIMD) pull (key tile, KV head)
//     units from per-XCD counters; the list is sorted longest-first;
//   * a unit = 128 keys of one segment of one work item for one KV head, looping over the query heads of the
//     KV head and over the 32-row query blocks ("steps") that see the tile.  The four waves of a SIMD own the
//     SAME 32 keys and split a step by ROLE, each role a short program of eight matrix instructions that fits
//     128 registers, so that four waves fit a SIMD and the hardware interleaves them (a wave's own matrix and
//     vector instructions hardly overlap on this chip; those of different waves of a SIMD do):
//       P wave:  S = Q K^T, P = exp2(c S - LSE log2 e) with the mask; keeps the K fragments of its 32 keys; leaves
//                P in LDS in bf16 operand form;
//       dS wave: dP - delta = dO V^T with the accumulator started at -delta; keeps the V fragments of its 32
//                keys; then, one step behind, dS = P o (dP - delta), left in LDS in bf16 operand form;
//       dV wave: dV += P^T dO, two steps behind, for 64 keys (those of two P waves) x 64 channels, so that every
//                transposed dO fragment read from LDS feeds two matrix instructions; P is the A operand and the
//                accumulator comes out as [key x channel] with the channel on the lane;
//       dK wave: dK += dS^T Q, three steps behind, 64 keys x 64 channels likewise;
//     one block barrier per step orders the hand-overs and the reuse of the LDS stages.  LDS bandwidth, not the
//     matrix pipe, bounds this kernel (about 1 KB of fragments per matrix instruction when a fragment is used
//     once), hence bf16 hand-overs and the 64 x 64 blocks of the accumulating waves;
//   * Q, dO blocks (32 rows) and their row statistics stream through LDS in five stages (two steps ahead, two
//     behind) filled by LDS-direct buffer loads, one tile instruction per wave and step; the tiles are
//     chunk-permuted so that both the row reads (A operands of S and dP) and the transpose reads (B operands
//     dO, Q of the accumulating contractions, one channel per lane) run at the full LDS rate;
//   * S and dP come out as [query x key] with the key on the lane, which is exactly the A-operand layout of
//     P^T and dS^T in dV += P^T dO and dK += dS^T Q: the hand-over is lane to same lane;
//   * inside the matrix phases every LDS fragment is requested several MFMAs before its use;
//   * the caller's fp32 accumulators: when the scheduler found that no other item of the launch touches the tile's
//     keys, the waves' accumulators start from the caller's values and the epilogue stores whole 128-byte lines;
//     otherwise they start at zero and the epilogue adds with fp32 atomics.
#include "fcp_bwd.h"

namespace fcp {
namespace {

template <int D>
struct DkvCfg {
  static constexpr int BN = kBwdBN;                // 128 keys per unit (32 per SIMD)
  static constexpr int BM = kBwdBM;                // 32 query rows per step
  static constexpr int NWAVE = 16;
  using DT = DualTile<D>;
  static constexpr int TILE = DT::bytes(BM);       // one Q or dO block
  static constexpr int SLOT = 256;                 // one statistics plane of a step: 64 floats (32 used)
  static constexpr int STAGE = 2 * TILE + 2 * SLOT;   // Q, dO, -LSE log2 e, -delta
  static constexpr int FILL_AHEAD = 2;             // steps between a block's fill and its first use
  static constexpr int NSTAGE = 3 + FILL_AHEAD;    // two steps behind, the step itself, FILL_AHEAD steps ahead
  // hand-over buffers of one key group, each double-buffered by step parity
  static constexpr int PB = 32 * 32 * 2;           // P or dS in bf16, B-operand form (2 x 16 bytes per lane)
  static constexpr int XGROUP = 2 * PB + 2 * PB;
  static constexpr int XOFF = NSTAGE * STAGE;
  static constexpr int LDS_BYTES = XOFF + 4 * XGROUP;
  static constexpr int NS = D / 16;                // MFMAs of one 32 x 32 block of S or dP
  static constexpr int NVA = D / 64;               // 32-channel blocks of dK^T / dV^T per accumulating wave (half of the channels)
  static constexpr int TINST = 2 * BM / DT::RPI;   // tile fill instructions per step (Q then dO), one per wave
  static constexpr int kAhead = 4;                 // LDS fragments requested this many MFMAs ahead
  static constexpr int DRAIN = 3;                  // iterations after the last step's contraction (the dK wave's lag)
  static_assert(TINST <= NWAVE, "one tile instruction per wave");
  static_assert(LDS_BYTES <= 160 * 1024, "LDS");
};

template <int D>
__global__ __launch_bounds__(1024, 1) void dkv_kernel(const BwdParams p) {
  using C = DkvCfg<D>;
  using DT = typename C::DT;
  extern __shared__ __attribute__((aligned(256))) unsigned char smem[];
  __shared__ int32_t s_next_unit;
  __shared__ int32_t s_rec[16];

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int role = wave >> 2;                     // 0: P, 1: dV, 2: dS, 3: dK
  // the producing waves go first at their SIMD's issue port: the accumulating waves' steps wait for what they make
  if (role == 0 || role == 2) __builtin_amdgcn_s_setprio(2);
  const int pw = wave & 3;                        // key group (and SIMD): keys 32 pw .. 32 pw + 31
  const int l32 = lane & 31, g2 = lane >> 5;
  const int G = p.hq / p.hkv;
  const uint32_t lds0 = lds_offset(smem);
  const bool per_xcd = (p.hkv % kNumXcd) == 0;
  const int xcd = per_xcd ? (int)(blockIdx.x % kNumXcd) : 0;
  const int kvh_here = per_xcd ? p.hkv / kNumXcd : p.hkv;
  UnitQueue uq;
  uq.init(p.hdr, p.tiles, xcd, kvh_here, &s_next_unit, s_rec);

  // ---- per-wave fill duty: tile instruction `wave` (the first half of the instructions fills Q, the second dO;
  // instruction j covers block rows RPI (j % (TINST/2)) ..) and, for two of the waves, one statistics plane
  const int q_row_bytes = p.hq * D * 2;
  const bool fill_tile = wave < C::TINST;
  const bool fill_is_do = wave >= C::TINST / 2;
  const int fill_row0 = DT::RPI * (wave % (C::TINST / 2));
  int tfill;
  {
    const int row = fill_row0 + lane / DT::CPR;
    tfill = row * q_row_bytes + (((lane % DT::CPR) ^ DT::key(row)) << 4);
  }
  const int stat_plane = (wave - C::TINST) & (C::NWAVE - 1);     // 0, 1: this wave loads that plane
  const bool fill_stat = stat_plane < 2;

  unsigned char* const xg = smem + C::XOFF + pw * C::XGROUP + lane * 16;
  unsigned char* const x_pb = xg;                       // + parity * PB + j * 1024, j < 2
  unsigned char* const x_ds = xg + 2 * C::PB;
  for (;;) {
    const int unit = uq.current(&s_next_unit);
    if (unit >= uq.n_units) break;
    const KTile t = read_record<KTile, 15>(s_rec);
    const int kvh = xcd * kvh_here + unit % kvh_here;
    uq.prefetch();

    const bool exclusive = (t.flags & kFlagSeg0Exclusive) != 0;
    const int n_keys = t.n_keys;                               // >= 1 by construction
    const int my_key = 32 * pw + l32;
    const int my_key_ld = min(my_key, n_keys - 1);
    const bool my_key_valid = my_key < n_keys;
    const int64_t kv_row0 = t.kv_row0;

    // query blocks that see the tile: from the block holding the first row that sees the tile's first key
    const int first_row = max(0, t.from_first[0] - t.q_seq_start);
    const int qb0 = first_row / C::BM;
    const int nqb = (t.q_len + C::BM - 1) / C::BM - qb0;       // query blocks per head, >= 1
    const int n_iter = nqb * G;

    // ---- fills ---------------------------------------------------------------------------------
    // Step s = (query head s / nqb of the KV head, query block qb0 + s % nqb).  The running state below names
    // the NEXT step to be filled; steps are filled strictly in order, the same loads in every call (past the last
    // step they fall outside the empty resources' range), which the vmcnt waits rely on.  Rows past the item's
    // last row lie outside the range and arrive as zeros.
    const int q_bytes = (t.q_len - 1) * q_row_bytes + D * 2;
    const int64_t plane = (int64_t)p.hq * p.tq;               // floats per statistics plane
    int f_head = kvh * G, f_left = nqb, f_heads_left = G;
    int f_soff = qb0 * C::BM * q_row_bytes, f_ssoff = qb0 * C::BM * 4;
    auto f_resources = [&](bool live, i32x4& rt, i32x4& rst) {
      rt = buffer_rsrc((fill_is_do ? p.d_o : p.q) + ((int64_t)t.q_local_off * p.hq + f_head) * D, live ? q_bytes : 0);
      rst = buffer_rsrc(p.stats + (stat_plane & 1) * plane + (int64_t)f_head * p.tq + t.q_local_off, live ? t.q_len * 4 : 0);
    };
    i32x4 f_rt, f_rst;
    f_resources(true, f_rt, f_rst);
    uint32_t f_dst = lds0;
    auto fill_next = [&]() {
      if (f_left == 0) {          // next head of the group (or past the end: empty resources)
        --f_heads_left;
        ++f_head;
        f_left = nqb;
        f_soff = qb0 * C::BM * q_row_bytes;
        f_ssoff = qb0 * C::BM * 4;
        f_resources(f_heads_left > 0, f_rt, f_rst);
      }
      if (C::TINST == C::NWAVE || fill_tile) lds_fill_b128(f_rt, f_dst + (fill_is_do ? C::TILE : 0) + DT::row_base(fill_row0), tfill, f_soff);
      if (fill_stat) lds_fill_b32(f_rst, f_dst + 2 * C::TILE + (stat_plane & 1) * C::SLOT, lane * 4, f_ssoff);
      --f_left;
      f_soff += C::BM * q_row_bytes;
      f_ssoff += C::BM * 4;
      f_dst += C::STAGE;
      if (f_dst == lds0 + C::NSTAGE * C::STAGE) f_dst = lds0;
    };
    // all but the newest batch of this wave's fills have landed
    auto wait_fills = [&]() {
      // One wait for every wave (no branch on the wave's number of fills per step, 0..2): with at most
      // FILL_AHEAD - 1 loads in flight everything older than the newest FILL_AHEAD - 1 batches has landed; a wave
      // with two loads per step waits for a little more than it must.
      __builtin_amdgcn_s_waitcnt(0x0F70 | (C::FILL_AHEAD - 1));
    };

    // Iteration `it` of the n_iter + DRAIN of a unit: the P and dS waves work on step it, the dS wave's vector phase
    // on step it - 1, the dV wave on step it - 2, the dK wave on step it - 3 (both with operands requested in the
    // iteration before).  At the top every wave has waited for all
    // its fills but the newest batch (step it + 1) and met the others, so the blocks of steps it - 2 .. it are
    // in LDS, P of step it - 1 and dS of step it - 2 are in their buffers, and the stage of step it - 3, last
    // read by the dK wave in iteration it - 1, is free for the fills of step it + 2.
    // Geometry.  Step s is block j = s % nqb of its head (the running counter `j` below, one advance per step).  A
    // key group takes part in a block if it has keys in the tile and its first key is not after the block's last
    // row, which holds from a first block on (first_active); its probabilities need the causal mask before a
    // first block (first_unmasked) and always if the tile ends inside the group.  Both are found once per unit, so
    // that a step costs one compare instead of the positions of its rows.
    auto pick = [](const int32_t (&a)[4], int grp) { return grp == 0 ? a[0] : grp == 1 ? a[1] : grp == 2 ? a[2] : a[3]; };
    auto first_active = [&](int grp) {
      const int thr = pick(t.from_first, grp) - t.q_seq_start;  // first row of the sequence part that sees the group
      if (32 * grp >= n_keys || thr > t.q_len - 1) return nqb;  // never
      return max(0, (max(thr, 0) >> 5) - qb0);
    };
    auto first_unmasked = [&](int grp) {
      if (32 * grp + 32 > n_keys) return nqb;                   // always masked
      const int thr = pick(t.from_last, grp) - t.q_seq_start;   // first row that sees all of the group's keys
      return max(0, ((max(thr, 0) + 31) >> 5) - qb0);
    };
    int j = 0;
    auto next_block = [&]() { if (++j == nqb) j = 0; };
    const unsigned char* stage = smem;                        // stage of step `it`
    auto next_stage = [&](const unsigned char* s) { s += C::STAGE; return s == smem + C::NSTAGE * C::STAGE ? smem : s; };

    if (role == 0 || role == 2) {
      const int j_act = first_active(pw), j_unmasked = first_unmasked(pw);
      // The first fills go out before the wave's own loads so that their latencies overlap.
#pragma unroll
      for (int a = 0; a < C::FILL_AHEAD; ++a) fill_next();
      // own-key fragments, B operand (lane = key column): K for the P wave, V for the dS wave
      bf16x8 kvf[C::NS];
      int my_key_from = t.k_pos0 + my_key;            // position of the first query that sees the lane's key
      {
        if (p.k_from) my_key_from = p.k_from[kv_row0 + my_key_ld];
        const uint16_t* src = role == 0 ? p.k : p.v;
        const int64_t off = ((kv_row0 + my_key_ld) * p.hkv + kvh) * D + 8 * g2;
#pragma unroll
        for (int ks = 0; ks < C::NS; ++ks) kvf[ks] = *reinterpret_cast<const bf16x8*>(src + off + 16 * ks);
        // The fragments must have arrived before the step loop: the compiler, which does not see the fills, would
        // otherwise wait for "its" loads inside the loop with vmcnt(0), and that wait also covers every fill in
        // flight.
        __builtin_amdgcn_s_waitcnt(0x0F70);
      }
      // row fragments (A operands of S = Q K^T, dP = dO V^T): lane reads block row l32, chunk 2 ks + g2
      int rowaddr[C::NS];
#pragma unroll
      for (int ks = 0; ks < C::NS; ++ks) rowaddr[ks] = tile_off<DT>(l32, 2 * ks + g2);
      // S or dP - delta [32 rows x 32 own keys]; register i of the result is block row 8 (i/4) + 4 g2 + i%4, so
      // the four row statistics a lane needs per group of four registers are contiguous
      auto contract = [&](f32x16& sacc, const unsigned char* rtile) {
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
      };
      if (role == 0) {
        for (int it = 0; it < n_iter + C::DRAIN; ++it, stage = next_stage(stage)) {
          wait_fills();
          __syncthreads();
          fill_next();
          const int jb = j;
          next_block();
          if (it >= n_iter || jb < j_act) continue;
          const float* stat = reinterpret_cast<const float*>(stage + 2 * C::TILE) + 4 * g2;
          f32x4 nl[4];           // -LSE log2 e of the rows of the lane's registers
#pragma unroll
          for (int j = 0; j < 4; ++j) nl[j] = *reinterpret_cast<const f32x4*>(stat + 8 * j);
          f32x16 sacc = zero16();
          contract(sacc, stage);
          // P = exp2(c S - LSE log2 e) with the mask.  Rows past the item's last row need no mask: their Q, dO
          // and statistics arrive as zeros, so P = 1 there meets dO = 0 in dV and dP - delta = 0 in dS.  That
          // leaves the causal edge and the keys past the tile's last.
          const bool need_mask = jb < j_unmasked;
          f32x4 pr[4];
          if (need_mask) {
            // register i is block row 8 (i/4) + 4 g2 + i%4; it sees the lane's key from the row at position my_key_from on
            const int q_pos0 = t.q_seq_start + (qb0 + jb) * C::BM;
            int lo = (my_key_valid ? my_key_from - q_pos0 : 1 << 20) - 4 * g2;
            asm volatile("; masked variant" : "+v"(lo));
#pragma unroll
            for (int i = 0; i < 16; ++i) {
              const float e = __builtin_amdgcn_exp2f(fmaf(sacc[i], p.scale_log2, nl[i / 4][i % 4]));
              pr[i / 4][i % 4] = (8 * (i / 4) + (i % 4) < lo) ? 0.f : e;
            }
          } else {
#pragma unroll
            for (int i = 0; i < 16; ++i) pr[i / 4][i % 4] = __builtin_amdgcn_exp2f(fmaf(sacc[i], p.scale_log2, nl[i / 4][i % 4]));
          }
          bf16x8 pb[2];
#pragma unroll
          for (int i = 0; i < 16; ++i) pb[i / 8][i % 8] = (__bf16)pr[i / 4][i % 4];
#pragma unroll
          for (int j = 0; j < 2; ++j) *reinterpret_cast<bf16x8*>(x_pb + (it & 1) * C::PB + j * 1024) = pb[j];
        }
      } else {
        bool prev_active = false;
        f32x16 dpacc = zero16();   // dP - delta of step it - 1 at the top of iteration it
        for (int it = 0; it < n_iter + C::DRAIN; ++it, stage = next_stage(stage)) {
          wait_fills();
          __syncthreads();
          fill_next();
          const bool active = it < n_iter && j >= j_act;
          next_block();
          if (prev_active) {
            // dS = P o (dP - delta) of step it - 1, with P as the dV wave sees it (bf16)
            bf16x8 pin[2];
#pragma unroll
            for (int j = 0; j < 2; ++j) pin[j] = *reinterpret_cast<const bf16x8*>(x_pb + ((it - 1) & 1) * C::PB + j * 1024);
            bf16x8 dsb[2];
#pragma unroll
            for (int i = 0; i < 16; ++i) dsb[i / 8][i % 8] = (__bf16)((float)pin[i / 8][i % 8] * dpacc[i]);
#pragma unroll
            for (int j = 0; j < 2; ++j) *reinterpret_cast<bf16x8*>(x_ds + ((it - 1) & 1) * C::PB + j * 1024) = dsb[j];
          }
          if (active) {
            const float* stat = reinterpret_cast<const float*>(stage + 2 * C::TILE) + C::SLOT / 4 + 4 * g2;
#pragma unroll
            for (int j = 0; j < 4; ++j) {        // the accumulator starts at -delta of its rows
              const f32x4 nd = *reinterpret_cast<const f32x4*>(stat + 8 * j);
#pragma unroll
              for (int e = 0; e < 4; ++e) dpacc[4 * j + e] = nd[e];
            }
            contract(dpacc, stage + C::TILE);
          }
          prev_active = active;
        }
      }
    } else {
      // Accumulating waves: 64 keys (the key groups 2 kp, 2 kp + 1 of two P / dS waves) x 64 channels (half ch).
      const int kp = pw >> 1, ch = pw & 1;
      const int j_act0 = first_active(2 * kp), j_act1 = first_active(2 * kp + 1);
      // transposed fragments (B operands dO, Q [query x channel], one channel per lane; k-slots = query rows 16 t + {4 g2 + [0,4),
      // 8 + 4 g2 + [0,4)}): inside a 16-lane block lane i supplies the address of block row (i / 4), channels
      // 4 (i % 4) + [0,4); block b covers channels 16 (b % 2) + [0,16) for row group b / 2
      int traddr[2][C::NVA];
      {
        const int row0 = 4 * g2 + ((lane & 15) >> 2);
        const int chunk0 = 2 * ((lane >> 4) & 1) + ((lane & 3) >> 1);
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
          for (int db = 0; db < C::NVA; ++db)
            traddr[h][db] = tile_off<DT>(row0 + 8 * h, 4 * (C::NVA * ch + db) + chunk0) + 8 * (lane & 1);
      }
#pragma unroll
      for (int a = 0; a < C::FILL_AHEAD; ++a) fill_next();
      // dV or dK [32-channel block][key group of the pair] as [key x channel]: the channel is on the lane, register i
      // is key 8 (i/4) + 4 g2 + i%4 of the group, so that a wave-wide access covers whole 128-byte lines of two keys.
      // When no other item of the launch touches the tile's keys the accumulators START at the caller's values
      // (divided by the factor that the epilogue applies) and the epilogue only stores.  The keys are reached
      // through a buffer resource that ends with the tile's last key (reads past it give zero, writes are
      // dropped): per-lane offset = the lane's part (key 4 g2 of a group of eight, channel l32), scalar offset = the
      // rest.
      f32x16 acc[C::NVA][2];
      const float mul = role == 1 ? 1.f : p.scale;
      const int row_bytes = p.hkv * D * 4;
      const int n_pair_keys = n_keys - 64 * kp;                    // keys of the tile in this wave's 64-key half
      const __amdgpu_buffer_rsrc_t racc = __builtin_amdgcn_make_buffer_rsrc(
          (void*)((role == 1 ? p.dv : p.dk) + ((kv_row0 + 64 * kp) * p.hkv + kvh) * D + 32 * C::NVA * ch), (short)0,
          n_pair_keys > 0 ? (n_pair_keys - 1) * row_bytes + 32 * C::NVA * 4 : 0, 0x00020000);
      const int acc_voff = 4 * g2 * row_bytes + 4 * l32;
      auto acc_soff = [&](int kb, int db, int i) { return (32 * kb + 8 * (i / 4) + (i % 4)) * row_bytes + 128 * db; };
      // Direct mode: the unit owns its keys, so nothing is read and the epilogue writes the final bf16 rows.
      const bool direct = exclusive && p.dk_out != nullptr;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int db = 0; db < C::NVA; ++db) {
          acc[db][kb] = zero16();
          if (exclusive && !direct) {
#pragma unroll
            for (int i = 0; i < 16; ++i)
              acc[db][kb][i] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(racc, acc_voff, acc_soff(kb, db, i), 0));
          }
        }
      // (explicit wait: the compiler must not be left to wait for these loads inside the step loop)
      __builtin_amdgcn_s_waitcnt(0x0F70);
      if (exclusive && !direct && role != 1) {
        const float inv = 1.f / p.scale;
#pragma unroll
        for (int db = 0; db < C::NVA; ++db)
#pragma unroll
          for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[db][kb][i] *= inv;
      }
      // The dV wave runs two steps behind the P wave, the dK wave three: their operands are complete one barrier
      // before they are used, so they are requested from LDS at the END of the iteration before (the LDS is then
      // not serving the burst of requests that follows a barrier) and the matrix instructions start right after
      // the barrier.
      const int lag = role == 1 ? 2 : 3;
      // B operands of a step, left by the pair's P / dS waves (same lane, key group 2 kp + kb)
      const unsigned char* const xb = smem + C::XOFF + (2 * kp) * C::XGROUP + lane * 16 + (role == 1 ? 0 : 2 * C::PB);
      const int tsel = role == 1 ? C::TILE : 0;                    // dO^T for dV, Q^T for dK
      // the stage of step it + 1 - lag (the step whose operands iteration `it` requests)
      const unsigned char* lstage = smem + (C::NSTAGE + 1 - lag) * C::STAGE;
      constexpr int N = 2 * C::NVA;                                // fragments: (tt, db)
      bf16x8 bop[2][2] = {}, fr[N] = {};                           // operands of the step of the next iteration
      bool have = false, act0 = false, act1 = false;
      for (int it = 0; it < n_iter + C::DRAIN; ++it, lstage = next_stage(lstage)) {
        // the requests of the last iteration have been served: their sources may be overwritten after the barrier
        __builtin_amdgcn_s_waitcnt(0xC07F);
        wait_fills();
        __syncthreads();
        fill_next();
        if (have) {
          // acc += P^T dO (dS^T Q): k-step tt of a P (dS) operand covers block rows 16 tt .. 16 tt + 15.  A group that
          // was not active left nothing in its buffer: its operand is zero.
          if (!(act0 && act1)) {     // rare (causal edge, tails): kept off the common path
#pragma unroll
            for (int tt = 0; tt < 2; ++tt) {
              if (!act0) bop[0][tt] = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
              if (!act1) bop[1][tt] = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
            }
          }
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int x = 0; x < N; ++x)
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
              acc[x % C::NVA][kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bop[kb][x / C::NVA], fr[x], acc[x % C::NVA][kb], 0, 0, 0);
              __builtin_amdgcn_sched_barrier(0);
            }
        }
        // requests for step s1 = it + 1 - lag: P of step s1 was written in iteration s1 <= it - 1 and dS of step s1 in
        // iteration s1 + 1 <= it - 1, so both are visible since this iteration's barrier
        const int s1 = it + 1 - lag;
        have = false;
        if (s1 >= 0) {
          if (s1 < n_iter) {
            act0 = j >= j_act0;
            act1 = j >= j_act1;
            have = act0 || act1;
          }
          next_block();
        }
        // (requested unconditionally: the addresses are valid LDS addresses for any s1, and registers that are
        // written in every iteration need no copies around the loop)
        {
#pragma unroll
          for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int tt = 0; tt < 2; ++tt)
              bop[kb][tt] = *reinterpret_cast<const bf16x8*>(xb + kb * C::XGROUP + (s1 & 1) * C::PB + tt * 1024);
          const unsigned char* ttile = lstage + tsel;
#pragma unroll
          for (int x = 0; x < N; ++x) {
            const unsigned char* b0 = ttile + (x / C::NVA) * (16 * DT::row_base(1));
            fr[x] = tr_read_8(b0 + traddr[0][x % C::NVA], b0 + traddr[1][x % C::NVA]);
          }
        }
      }
      // epilogue: dV or dK [key x channel] -> pool accumulators (or, in direct mode, the final bf16 rows: half a line
      // per store)
      if (direct) {
        const int out_row_bytes = p.hkv * D * 2;
        const __amdgpu_buffer_rsrc_t rout = __builtin_amdgcn_make_buffer_rsrc(
            (void*)((role == 1 ? p.dv_out : p.dk_out) + ((kv_row0 + 64 * kp) * p.hkv + kvh) * D + 32 * C::NVA * ch), (short)0,
            n_pair_keys > 0 ? (n_pair_keys - 1) * out_row_bytes + 32 * C::NVA * 2 : 0, 0x00020000);
        const int out_voff = 4 * g2 * out_row_bytes + 2 * l32;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int db = 0; db < C::NVA; ++db)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
              const __bf16 val = (__bf16)(acc[db][kb][i] * mul);
              __builtin_amdgcn_raw_buffer_store_b16(__builtin_bit_cast(short, val), rout, out_voff,
                                                    (32 * kb + 8 * (i / 4) + (i % 4)) * out_row_bytes + 64 * db, 0);
            }
      } else {
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int db = 0; db < C::NVA; ++db)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
              const float val = acc[db][kb][i] * mul;
              if (exclusive) __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, val), racc, acc_voff, acc_soff(kb, db, i), 0);
              else __builtin_amdgcn_raw_ptr_buffer_atomic_fadd_f32(val, racc, acc_voff, acc_soff(kb, db, i), 0);
            }
      }
    }
    uq.advance(&s_next_unit, s_rec);   // barrier: the LDS stages are free for the next unit's fills
  }
}

}  // namespace

int launch_dkv(const BwdParams& p, int head_dim, int64_t units, int n_cu, hipStream_t stream) {
  int64_t blocks = n_cu;                               // one 1024-thread block per CU
  if (blocks > units) blocks = (units + 7) / 8 * 8;   // a multiple of the XCD count
  if (blocks < 8) blocks = 8;
  static std::atomic<uint64_t> lds_done[2];
  int rc;
  if (head_dim == 128) {
    if ((rc = raise_lds_limit((const void*)dkv_kernel<128>, DkvCfg<128>::LDS_BYTES, lds_done[0])) != FCP_OK) return rc;
    hipLaunchKernelGGL(dkv_kernel<128>, dim3((unsigned)blocks), dim3(1024), DkvCfg<128>::LDS_BYTES, stream, p);
  } else {
    if ((rc = raise_lds_limit((const void*)dkv_kernel<64>, DkvCfg<64>::LDS_BYTES, lds_done[1])) != FCP_OK) return rc;
    hipLaunchKernelGGL(dkv_kernel<64>, dim3((unsigned)blocks), dim3(1024), DkvCfg<64>::LDS_BYTES, stream, p);
  }
  FCP_HIP_CHECK(hipGetLastError());
  return FCP_OK;
}

}  // namespace fcp
