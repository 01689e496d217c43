// fcp_attn_bwd_step: gradient contributions of one CP rank for its ring steps.
//
// Backward of O = softmax(scale Q K^T) V (paper Eq. 1, Sec. 3.1; causal mask, Sec. 4.3) for
// the key sets the ring steps bring (ring-style CP, Sec. 3.2).  With the merged LSE the
// probabilities of a step are recomputed exactly, P = exp(scale s - LSE), so each step adds
// its own share:  dV += P^T dO,  dS = P o (dO V^T - delta),  dQ += scale dS K,  dK += scale dS^T Q.
//
// gfx950 design: two persistent kernels (dK/dV over key tiles in its own file, dQ here), because fp32 atomics
// retire at about one element per L2 channel per clock on this chip (~270 G/s), far too few to accumulate dQ
// per key tile.
//
// dq_kernel: persistent 512-thread blocks (8 wave64, one block per CU, two waves per SIMD, up to 256 registers each) pull
// units from per-XCD counters.  A unit = 128 query rows of one work item for TWO query heads of one KV head (waves
// 0..3 the first head, waves 4..7 the second), or, when the heads per KV head are odd, 256 rows for one head; either
// way the eight waves share every K / V block, looping over the 32-key blocks ("steps") of the two key segments that
// the rows see.  K and V blocks stream through LDS in four stages filled by LDS-direct buffer loads; the tiles are
// chunk-permuted so that both row reads and transpose reads run at the full LDS rate.  The waves are INDEPENDENT: each
// owns 32 query rows (Q and dO fragments in registers, one query per lane, so LSE, delta and the causal bound are
// per-lane constants) and does everything for them, so nothing is handed from wave to wave and the only block-wide
// meeting is the one barrier per step that recycles the LDS stages.  Per step and wave:
//   A  S^T = K Q^T and dP^T = V dO^T [key x query] for the step's 32 keys (row reads of K and V),
//   V  P^T = exp2(c S^T - LSE log2 e) with the mask, dS^T = P^T o (dP^T - delta), bf16, in registers in the A-operand form of
//   Q  dQ += dS K [query x channel] (K^T by transpose reads).
// A single wave issues about one instruction every six cycles whatever its kind, so the vector work of one wave has to
// meet the matrix work of ANOTHER wave of its SIMD: waves w and w + 4 share a SIMD, and a step is two slots, as in the
// forward kernel - a matrix slot (Q of step it - 1, its transposed fragments requested before the slot's barrier, then
// A of step it: 24 matrix instructions back to back, at raised priority) and a vector slot (V of step it); waves 4..7
// run one slot behind waves 0..3 (one barrier more at the start of a unit, one less at its end), so that the matrix
// slot of one wave meets the vector slot of the other.
// (Two predecessors: a role-split kernel - P, dS and dQ waves exchanging bf16 tiles through LDS, 12 waves - spent its
// steps in the hand-over chain barrier -> LDS -> matrix -> exponentials -> LDS -> barrier; the same independent waves
// with ONE barrier per step and the second group's parts merely reordered (V Q of step it - 1, then A of step it) left
// the two waves of a SIMD competing for the matrix pipe in one phase and idle at the barrier in another: 7 % slower
// on a 16384-token sequence, 4 % on the packed workload.)
// The result is added to the caller's fp32 accumulator once per unit: with plain
// load-add-store when the scheduler found that no other item of the launch touches the same rows (always the
// case for degree-1 sequences), otherwise with fp32 atomics.
#include "fcp_bwd.h"

#include <type_traits>

namespace fcp {
namespace {

template <int D>
struct DqCfg {
  static constexpr int BK = kDqBN;                 // keys per step
  static constexpr int NWAVE = 8;
  using DT = DualTile<D>;
  static constexpr int TILE = DT::bytes(BK);       // one K or V block
  static constexpr int STAGE = 2 * TILE;           // K, V
  static constexpr int FILL_AHEAD = 2;             // steps between a block's fill and its first use
  static constexpr int NSTAGE = 2 + FILL_AHEAD;    // one step behind (the second wave group), the step itself, FILL_AHEAD ahead
  static constexpr int AREA = RowTile<D>::bytes(32);   // per wave: its 32 rows of Q, then of dO, on their way in
  static constexpr int LDS_BYTES = NSTAGE * STAGE + NWAVE * AREA;
  static constexpr int NS = D / 16;                // k-steps of one 32 x 32 block of S^T or dP^T
  static constexpr int NCB = D / 32;               // 32-channel blocks of dQ
  static constexpr int TINST = 2 * BK / DT::RPI;   // tile fill instructions per step (K then V)
  static constexpr int IPW = TINST / NWAVE;        // ... per wave: waves 0..3 fill K, waves 4..7 fill V
  static constexpr int NQ = 2 * NCB;               // matrix instructions of a step's accumulation
  static constexpr int kAhead = 4;                 // row fragments requested this many matrix instructions ahead (6: registers spill)
  static_assert(IPW * NWAVE == TINST && IPW >= 1, "fill split");
  static_assert(BK == 32, "one 32 x 32 score block per wave and step");
};

template <int D>
__global__ __launch_bounds__(512, 1) void dq_kernel(const BwdParams p, const int head_pair) {
  using C = DqCfg<D>;
  using DT = typename C::DT;
  extern __shared__ __attribute__((aligned(256))) unsigned char smem[];
  __shared__ int32_t s_next_unit;
  __shared__ int32_t s_rec[16];

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int grp = wave >> 2;                      // 0: waves 0..3, 1: waves 4..7 (the shifted group)
  const int l32 = lane & 31, g2 = lane >> 5;
  const int G = p.hq / p.hkv;
  const uint32_t lds0 = lds_offset(smem);
  // unit numbering: when the heads split evenly each XCD owns a contiguous eighth of them (so the K/V of a KV head stay
  // in one L2); a unit covers one head or, in head-pair mode, two consecutive heads
  const int hpu = head_pair ? 2 : 1;
  const bool per_xcd = (p.hq % (kNumXcd * hpu)) == 0;
  const int xcd = per_xcd ? (int)(blockIdx.x % kNumXcd) : 0;
  const int heads_here = per_xcd ? p.hq / kNumXcd : p.hq;
  const int units_per_tile = heads_here / hpu;
  UnitQueue uq;
  uq.init(p.hdr, p.tiles, xcd, units_per_tile, &s_next_unit, s_rec);

  // ---- per-wave fill duty: IPW tile instructions of K (waves 0..3) or of V (waves 4..7); instruction j of a block
  // covers its rows RPI j ..  (the chunk permutation depends on the rows, so every instruction has its own offsets)
  const int kv_row_bytes = p.hkv * D * 2;
  const bool fill_is_v = wave >= 4;
  int tfill[C::IPW], fill_dst[C::IPW];
#pragma unroll
  for (int i = 0; i < C::IPW; ++i) {
    const int row0 = DT::RPI * (C::IPW * (wave & 3) + i);
    const int row = row0 + lane / DT::CPR;
    tfill[i] = row * kv_row_bytes + (((lane % DT::CPR) ^ DT::key(row)) << 4);
    fill_dst[i] = (fill_is_v ? C::TILE : 0) + DT::row_base(row0);
  }
  // row fragments (A operands of S^T = K Q^T, dP^T = V dO^T): lane reads block row (key) l32, chunk 2 ks + g2
  int rowaddr[C::NS];
#pragma unroll
  for (int ks = 0; ks < C::NS; ++ks) rowaddr[ks] = tile_off<DT>(l32, 2 * ks + g2);
  // transposed fragments of the K block (B operand K [key x channel], one channel per lane; k-slots = keys 16 t + {4 g2 + [0,4),
  // 8 + 4 g2 + [0,4)}): inside a 16-lane block lane i supplies the address of block row (i / 4), channels
  // 4 (i % 4) + [0,4); block b covers channels 16 (b % 2) + [0,16) for row group b / 2
  int traddr[2][C::NCB];
  {
    const int row0 = 4 * g2 + ((lane & 15) >> 2);
    const int chunk0 = 2 * ((lane >> 4) & 1) + ((lane & 3) >> 1);
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
      for (int db = 0; db < C::NCB; ++db) traddr[h][db] = tile_off<DT>(row0 + 8 * h, 4 * db + chunk0) + 8 * (lane & 1);
  }

  for (;;) {
    const int unit = uq.current(&s_next_unit);
    if (unit >= uq.n_units) break;
    const QTile t = read_record<QTile, 12>(s_rec);
    const int head = xcd * heads_here + (unit % units_per_tile) * hpu + (head_pair ? grp : 0);
    const int kvh = head / G;

    const bool exclusive = (t.flags & kFlagQExclusive) != 0;
    const int rows_here = t.rows;
    // the two segments' fields as scalars: indexing the record's arrays with a run-time segment number would put
    // the record into scratch memory, and a scratch load inside the step loop waits with vmcnt(0), fills included
    const int vis0 = t.vis[0], vis1 = t.vis[1], kpos0 = t.k_pos0[0], kpos1 = t.k_pos0[1];
    const int64_t kvrow0 = t.kv_row0[0], kvrow1 = t.kv_row0[1];
    const int nt0 = (vis0 + C::BK - 1) / C::BK, nt1 = (vis1 + C::BK - 1) / C::BK;
    const int n_iter = nt0 + nt1;

    // ---- fills ---------------------------------------------------------------------------------
    // Step s = key block s of segment 0 for s < nt0, else block s - nt0 of segment 1.  The running state names
    // the NEXT step to be filled; the same loads in every call (past the last step they fall outside the empty
    // resources' range), which the vmcnt waits rely on.  Keys past the segment's visible part lie outside the
    // range and arrive as zeros.
    int f_seg = nt0 > 0 ? 0 : 1, f_left = nt0 > 0 ? nt0 : nt1, f_soff = 0;
    auto f_resource = [&](int seg, bool live) {
      const uint16_t* base = (fill_is_v ? p.v : p.k) + ((seg ? kvrow1 : kvrow0) * p.hkv + kvh) * D;
      return buffer_rsrc(base, live ? ((seg ? vis1 : vis0) - 1) * kv_row_bytes + D * 2 : 0);
    };
    i32x4 f_r = f_resource(f_seg, n_iter > 0);
    uint32_t f_dst = lds0;
    auto fill_next = [&]() {
      if (f_left == 0) {          // segment 1 (or past the end: empty resources)
        const bool live = f_seg == 0 && nt1 > 0;
        f_seg = 1;
        f_left = live ? nt1 : (1 << 30);
        f_soff = 0;
        f_r = f_resource(1, live);
      }
#pragma unroll
      for (int i = 0; i < C::IPW; ++i) lds_fill_b128(f_r, f_dst + fill_dst[i], tfill[i], f_soff);
      --f_left;
      f_soff += C::BK * kv_row_bytes;
      f_dst += C::STAGE;
      if (f_dst == lds0 + C::NSTAGE * C::STAGE) f_dst = lds0;
    };
    // all but the newest batch of this wave's fills have landed
    auto wait_fills = [&]() { __builtin_amdgcn_s_waitcnt(0x0F70 | C::IPW); };

    // Geometry.  Step s < nt0 is key block s of segment 0, step s >= nt0 block s - nt0 of segment 1; inside a segment
    // the key positions grow with the step.  The wave's rows take part in the leading blocks of a segment (those whose
    // first key the group's last row still sees) and need no mask in the leading blocks that all its rows see in
    // full; both counts are found once per unit, so that a step costs a few compares instead of its positions.
    const int wave_r0 = 32 * (head_pair ? (wave & 3) : wave);
    const int my_row = wave_r0 + l32;
    const int row_ld = min(my_row, rows_here - 1);
    int a0 = 0, b1 = 0, u0 = 0, u1 = 0;     // active: s < a0 or nt0 <= s < b1; unmasked: s < u0 or nt0 <= s < u1
    if (wave_r0 < rows_here) {
      // last key position seen by the group's first and by its last row (the limits grow with the row)
      int first = t.q_pos0 + wave_r0, last = t.q_pos0 + min(wave_r0 + 31, rows_here - 1);
      if (p.q_limit) {
        first = p.q_limit[t.q_row0 + wave_r0];
        last = p.q_limit[t.q_row0 + min(wave_r0 + 31, rows_here - 1)];
      }
      auto count = [&](int kpos, int vis, int nt, int& act, int& unm) {
        act = last >= kpos ? min(nt, ((last - kpos) >> 5) + 1) : 0;                 // blocks with kpos + 32 kt <= last
        const int full = first - kpos - 31 >= 0 ? ((first - kpos - 31) >> 5) + 1 : 0;   // ... with kpos + 32 kt + 31 <= first
        unm = min(full, vis / C::BK);                                              // and all 32 keys valid
      };
      int a1, v1;
      count(kpos0, vis0, nt0, a0, u0);
      count(kpos1, vis1, nt1, a1, v1);
      b1 = nt0 + a1;
      u1 = nt0 + v1;
    }
    auto in_span = [&](int s, int lo_end, int hi_end) { return s >= 0 && (s < lo_end || (s >= nt0 && s < hi_end)); };

    // -LSE log2 e and -delta of the lane's row: asked for first, they arrive while the tiles below are on their way
    const float stat_p = p.stats[(int64_t)head * p.tq + t.q_row0 + row_ld];
    const float stat_d = p.stats[(int64_t)p.hq * p.tq + (int64_t)head * p.tq + t.q_row0 + row_ld];
    // The first fills go out before the wave's own loads so that their latencies overlap.
#pragma unroll
    for (int a = 0; a < C::FILL_AHEAD; ++a) fill_next();
    // own-row fragments, B operands (lane = query column), channels 16 ks + 8 g2 + [0,8): Q and dO.  Loaded straight
    // from global memory in that form, every instruction would touch 32 cache lines for 32 bytes of each and a unit's
    // start would be bound by the rate of the address pipeline (several microseconds for the block's 128 KB); instead
    // the wave's 32 rows come in whole (LDS-direct fills of four rows each) through its staging area, one tensor after
    // the other, and the fragments are read from there.  Rows past the tile's last arrive as zeros.
    const int n_wave_rows = rows_here - wave_r0;                 // rows of the tile from this wave's first on
    bf16x8 qf[C::NS], dof[C::NS];
    {
      using RT = RowTile<D>;
      int lane_p = lane;                            // addresses formed here, not ahead of the unit loop (registers)
      asm volatile("" : "+v"(lane_p));
      const int q_row_bytes = p.hq * D * 2;
      const int64_t base = ((int64_t)(t.q_row0 + wave_r0) * p.hq + head) * D;
      const int nbytes = n_wave_rows > 0 ? (min(n_wave_rows, 32) - 1) * q_row_bytes + D * 2 : 0;
      const int area = C::NSTAGE * C::STAGE + wave * C::AREA;
      auto load_tile = [&](const uint16_t* src, bf16x8 (&f)[C::NS]) {
        const i32x4 r = buffer_rsrc(src + base, nbytes);
#pragma unroll
        for (int i = 0; i < 32 / RT::RPI; ++i)
          lds_fill_b128(r, lds0 + area + RT::row_base(RT::RPI * i), fill_voff<RT>(32, 0, i, lane_p, q_row_bytes), 0);
        __builtin_amdgcn_s_waitcnt(0x0F70);         // vmcnt(0)
#pragma unroll
        for (int ks = 0; ks < C::NS; ++ks)
          f[ks] = *reinterpret_cast<const bf16x8*>(smem + area + tile_off<RT>(lane_p & 31, 2 * ks + (lane_p >> 5)));
        __builtin_amdgcn_s_waitcnt(0xC07F);         // lgkmcnt(0): in registers before the area is filled again
      };
      load_tile(p.q, qf);
      load_tile(p.d_o, dof);
    }
    int q_lim = t.q_pos0 + my_row;                 // last key position the lane's row sees
    if (p.q_limit) q_lim = p.q_limit[t.q_row0 + row_ld];
    // dQ [32-channel block] as [query x channel]: the channel is on the lane, register i is row 8 (i/4) + 4 g2 + i%4 of
    // the wave's 32, so that a wave-wide access covers whole 128-byte lines of two rows.
    // When no other item of the launch touches the tile's rows the accumulators START at the caller's values
    // (divided by the scale that the epilogue applies) and the epilogue only stores.
    // The rows are reached through a buffer resource that ends with the tile's last row (reads past it give zero,
    // writes are dropped): per-lane offset = the lane's part (row 4 g2 of a group of eight, channel l32), scalar
    // offset = the rest.
    f32x16 acc[C::NCB];
    const int row_bytes = p.hq * D * 4;
    const __amdgpu_buffer_rsrc_t racc = __builtin_amdgcn_make_buffer_rsrc(
        (void*)(p.dq + ((int64_t)(t.q_row0 + wave_r0) * p.hq + head) * D), (short)0,
        n_wave_rows > 0 ? (n_wave_rows - 1) * row_bytes + D * 4 : 0, 0x00020000);
    const int acc_voff = 4 * g2 * row_bytes + 4 * l32;
    auto acc_soff = [&](int db, int i) { return (8 * (i / 4) + (i % 4)) * row_bytes + 128 * db; };
    // Direct mode: the unit owns its rows, so nothing is read and the epilogue writes the final bf16 rows.
    const bool direct = exclusive && p.dq_out != nullptr;
#pragma unroll
    for (int db = 0; db < C::NCB; ++db) {
      acc[db] = zero16();
      if (exclusive && !direct) {
#pragma unroll
        for (int i = 0; i < 16; ++i)
          acc[db][i] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(racc, acc_voff, acc_soff(db, i), 0));
      }
    }
    // These loads must have arrived before the step loop: the compiler, which does not see the fills, would
    // otherwise wait for them inside the loop with vmcnt(0), and that wait also covers every fill in flight.
    __builtin_amdgcn_s_waitcnt(0x0F70);
    if (exclusive && !direct) {
      const float inv_scale = 1.f / p.scale;
#pragma unroll
      for (int db = 0; db < C::NCB; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[db][i] *= inv_scale;
    }

    // ---- the step loop --------------------------------------------------------------------------------------------
    // Iteration `it` of n_iter + 1, two slots.  Before the first barrier the wave has waited for all its fills but the
    // newest batch (step it + 1), so after it the blocks of steps it - 1 and it are in LDS and the stage of step it - 2 is
    // free for step it + 2.  Matrix slot: Q(it - 1), A(it).  Vector slot: V(it), whose dS waits in registers for the next
    // matrix slot.  Waves 4..7 pass every barrier one slot later than waves 0..3, so they wait for their fills once more
    // before the second barrier: the waves 0..3 read the block of step it + 1 right after it.
    // Each of the three parts exists once in the program and is run or skipped as a whole (variants of the accumulating
    // part make the register allocator keep copies of the accumulators and move them in every step).
    f32x16 sacc = zero16(), dpacc = zero16();
    bf16x8 ds[2] = {};
    int st_a = 0;                                  // byte offset of the stage of step `it`
    int st_b = (C::NSTAGE - 1) * C::STAGE;         // ... of step it - 1
    auto bump = [&](int& s) { s += C::STAGE; if (s == C::NSTAGE * C::STAGE) s = 0; };
    // A: S^T and dP^T of the step whose blocks are at stage offset `so`
    auto part_a = [&](int so) {
      const unsigned char* const sa = smem + so;
      constexpr int NA = 2 * C::NS;
      bf16x8 fr[NA];
      auto req = [&](int z) { fr[z] = *reinterpret_cast<const bf16x8*>(sa + (z & 1) * C::TILE + rowaddr[z / 2]); };   // K (even) / V (odd), k-step z / 2
#pragma unroll
      for (int z = 0; z < C::kAhead; ++z) req(z);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int z = 0; z < NA; ++z) {
        if (z & 1) dpacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[z], dof[z / 2], z == 1 ? zero16() : dpacc, 0, 0, 0);
        else sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[z], qf[z / 2], z == 0 ? zero16() : sacc, 0, 0, 0);
        if (z + C::kAhead < NA) req(z + C::kAhead);
        __builtin_amdgcn_sched_barrier(0);
      }
    };
    // The vector part of step sv: P^T = exp2(c S^T - LSE log2 e), masked where the key is past the block's valid keys
    // or after the row; dS^T = P^T (dP^T - delta).  Register i is key 8 (i/4) + 4 g2 + i%4.
    auto part_v = [&](int sv) {
      if (in_span(sv, u0, u1)) {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const float e = __builtin_amdgcn_exp2f(fmaf(sacc[i], p.scale_log2, stat_p));
          ds[i / 8][i % 8] = (__bf16)(e * (dpacc[i] + stat_d));
        }
      } else {
        const bool seg1 = sv >= nt0;
        const int kt = sv - (seg1 ? nt0 : 0);
        const int k_pos0 = (seg1 ? kpos1 : kpos0) + kt * C::BK;
        const int n_valid = min(C::BK, (seg1 ? vis1 : vis0) - kt * C::BK);
        int hi = min(n_valid, q_lim - k_pos0 + 1) - 4 * g2;     // keys (minus 4 g2) below this bound are seen
        asm volatile("; masked variant" : "+v"(hi));
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const float e = __builtin_amdgcn_exp2f(fmaf(sacc[i], p.scale_log2, stat_p));
          ds[i / 8][i % 8] = (__bf16)((8 * (i / 4) + (i % 4) < hi) ? e * (dpacc[i] + stat_d) : 0.f);
        }
      }
    };
    // The transposed K fragments of the block at stage offset `so` (fragment (tt, db) = (x / NCB, x % NCB)) and the
    // accumulation dQ += dS K that uses them.
    bf16x8 tf[C::NQ] = {};
    auto tr_request = [&](int so) {
#pragma unroll
      for (int x = 0; x < C::NQ; ++x) {
        const unsigned char* b0 = smem + so + (x / C::NCB) * (16 * DT::row_base(1));
        tf[x] = tr_read_8(b0 + traddr[0][x % C::NCB], b0 + traddr[1][x % C::NCB]);
      }
    };
    auto part_q = [&]() {
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int x = 0; x < C::NQ; ++x) {
        acc[x % C::NCB] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ds[x / C::NCB], tf[x], acc[x % C::NCB], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);
      }
    };
    if (grp == 1) __syncthreads();
    for (int it = 0; it <= n_iter; ++it) {
      const bool q_on = in_span(it - 1, a0, b1);
      const bool a_on = it < n_iter && in_span(it, a0, b1);
      if (q_on) tr_request(st_b);
      wait_fills();
      __syncthreads();
      fill_next();
      __builtin_amdgcn_s_setprio(3);   // the matrix stream goes first at the SIMD's issue port (as in the forward kernel)
      if (q_on) part_q();
      if (a_on) part_a(st_a);
      __builtin_amdgcn_s_setprio(0);
      wait_fills();
      __syncthreads();
      if (a_on) part_v(it);
      bump(st_a);
      bump(st_b);
    }
    if (grp == 0) __syncthreads();

    // The next unit's record and the number of the unit after it start their trips here, ahead of the epilogue's
    // stores: the wave waits for the number (asked for one unit ago) in program order, and after the stores that wait
    // would last until the last of them has been written.
    uq.prefetch();
    // epilogue: dQ [query x channel] * scale -> accumulator rows (or, in direct mode, the final bf16 rows: half a
    // line per store).  Staging the tile through LDS for 16-byte stores of whole rows, as the forward kernel does,
    // measured slower here (+4 % on the packed workload): the narrow stores cost this wave only their issue.
    int lane_e = lane;                              // addresses formed here, not ahead of the unit's loop (registers)
    asm volatile("" : "+v"(lane_e));
    const int l32e = lane_e & 31, g2e = lane_e >> 5;
    if (direct) {
      const int out_row_bytes = p.hq * D * 2;
      const __amdgpu_buffer_rsrc_t rout = __builtin_amdgcn_make_buffer_rsrc(
          (void*)(p.dq_out + ((int64_t)(t.q_row0 + wave_r0) * p.hq + head) * D), (short)0,
          n_wave_rows > 0 ? (n_wave_rows - 1) * out_row_bytes + D * 2 : 0, 0x00020000);
      const int out_voff = 4 * g2e * out_row_bytes + 2 * l32e;
#pragma unroll
      for (int db = 0; db < C::NCB; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const __bf16 val = (__bf16)(acc[db][i] * p.scale);
          __builtin_amdgcn_raw_buffer_store_b16(__builtin_bit_cast(short, val), rout, out_voff,
                                                (8 * (i / 4) + (i % 4)) * out_row_bytes + 64 * db, 0);
        }
    } else {
#pragma unroll
      for (int db = 0; db < C::NCB; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const float val = acc[db][i] * p.scale;
          if (exclusive) __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, val), racc, acc_voff, acc_soff(db, i), 0);
          else __builtin_amdgcn_raw_ptr_buffer_atomic_fadd_f32(val, racc, acc_voff, acc_soff(db, i), 0);
        }
    }
    uq.advance(&s_next_unit, s_rec);   // barrier: the LDS stages are free for the next unit's fills
  }
}

}  // namespace
}  // namespace fcp

using fcp::fail;

// Both entry points; q_limit == k_from == NULL is the causal mask.
static int bwd_step(const void* q, const void* k, const void* v, const void* d_o, const float* lse,
                    const float* delta, const int32_t* cu_seqlens_kv, int32_t n_seqs,
                    const fcp_work_desc* work, int64_t n_work, int32_t tq, int32_t tkv, int32_t hq,
                    int32_t hkv, int32_t head_dim, float softmax_scale, const int32_t* q_limit, const int32_t* k_from,
                    float* dq_acc, float* dk_acc, float* dv_acc, void* scratch, size_t scratch_bytes, void* stream,
                    void* dq_out = nullptr, void* dk_out = nullptr, void* dv_out = nullptr) {
  fcp::clear_error();
  if (!q || !k || !v || !d_o || !lse || !delta || !cu_seqlens_kv || !dq_acc || !dk_acc || !dv_acc || !scratch)
    return fail(FCP_ERR_INVALID_ARG, "fcp_attn_bwd_step: null pointer");
  const bool direct = dq_out != nullptr;
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

  // The Q / dO rows of a work item are reached through one buffer resource with 32-bit byte offsets, which the fills
  // advance a few blocks past the item's end; an item has at most tq rows.  (The accumulators and outputs are reached
  // tile by tile, the pool segment by segment: the scheduler bounds a segment.)
  if ((int64_t)tq * hq * head_dim * 2 + ((int64_t)1 << 22) >= ((int64_t)1 << 31))
    return fail(FCP_ERR_UNSUPPORTED, "fcp_attn_bwd_step: tq * hq * head_dim must stay below 2^30 - 2^21 elements");
  hipStream_t st = (hipStream_t)stream;
  const int64_t cap_kv = fcp::kv_tile_cap(tkv, n_work);
  const int64_t cap_q = fcp::q_tile_cap(tq, tkv, n_work, 1 << 20);
  if (cap_kv > INT32_MAX / 64 || cap_q > INT32_MAX / 64) return fail(FCP_ERR_UNSUPPORTED, "fcp_attn_bwd_step: too many tiles");
  void* region_kv = scratch;
  void* region_q = static_cast<char*>(scratch) + fcp::sched_region_bytes(n_work, cap_kv);
  float* stats = reinterpret_cast<float*>(static_cast<char*>(region_q) + fcp::sched_region_bytes(n_work, cap_q));
  // direct mode: where every row's result comes from (and the accumulator rows that are accumulated into cleared),
  // on extra blocks of the scheduling launch
  fcp::RowStates rs{};
  if (direct) {
    rs.q_state = fcp::bwd_q_state(scratch, n_work, tq, tkv, hq);
    rs.kv_state = fcp::bwd_kv_state(scratch, n_work, tq, tkv, hq);
    rs.dq_acc = dq_acc; rs.dk_acc = dk_acc; rs.dv_acc = dv_acc;
    rs.q_row_elems = hq * head_dim; rs.kv_row_elems = hkv * head_dim;
    rs.n_parts = 1; rs.check_step = false;
  }
  if (tq == 0 || n_work == 0) {     // nothing to add; the lists are still built so that the status call works
    if (direct) {
      const int rcs = fcp::launch_row_states((int64_t)hkv * head_dim * 2, rs, q_limit, k_from, work, n_work, cu_seqlens_kv,
                                             n_seqs, tq, tkv, st);
      if (rcs != FCP_OK) return rcs;
    }
    int rc0 = fcp::launch_schedule(true, fcp::kBwdBN, fcp::kBwdBM, (int64_t)hkv * head_dim * 2, q_limit, k_from, work, n_work, cu_seqlens_kv, n_seqs, tq, tkv, 1, cap_kv, region_kv, nullptr, 0, st);
    if (rc0 != FCP_OK) return rc0;
    return fcp::launch_schedule(false, fcp::kDqBM, fcp::kDqBN, (int64_t)hkv * head_dim * 2, q_limit, k_from, work, n_work, cu_seqlens_kv, n_seqs, tq, tkv, 1, cap_q, region_q, nullptr, 0, st);
  }
  // dQ units: 128 query rows for two heads of one KV head when the heads pair up, else 256 rows for one head
  const int head_pair = ((hq / hkv) % 2 == 0) ? 1 : 0;
  int rc = fcp::launch_schedule_bwd((int64_t)hkv * head_dim * 2, q_limit, k_from, work, n_work, cu_seqlens_kv, n_seqs, tq, tkv,
                                    cap_kv, region_kv, head_pair ? fcp::kDqBM : 2 * fcp::kDqBM, cap_q, region_q, lse, delta, (int64_t)hq * tq, stats, st,
                                    direct ? &rs : nullptr);
  if (rc != FCP_OK) return rc;

  fcp::BwdParams p;
  p.q = (const uint16_t*)q; p.k = (const uint16_t*)k; p.v = (const uint16_t*)v; p.d_o = (const uint16_t*)d_o;
  p.lse = lse; p.delta = delta; p.stats = stats;
  p.q_limit = q_limit; p.k_from = k_from;
  p.dq = dq_acc; p.dk = dk_acc; p.dv = dv_acc;
  p.dq_out = (uint16_t*)dq_out; p.dk_out = (uint16_t*)dk_out; p.dv_out = (uint16_t*)dv_out;
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
  const int64_t dq_units = cap_q * (hq / (head_pair ? 2 : 1));
  if (head_dim == 128) {
    static std::atomic<uint64_t> lds_done;
    if ((rc = fcp::raise_lds_limit((const void*)fcp::dq_kernel<128>, fcp::DqCfg<128>::LDS_BYTES, lds_done)) != FCP_OK) return rc;
    hipLaunchKernelGGL(fcp::dq_kernel<128>, grid_for(dq_units, 1), dim3(512), fcp::DqCfg<128>::LDS_BYTES, st, p, head_pair);
  } else {
    static std::atomic<uint64_t> lds_done;
    if ((rc = fcp::raise_lds_limit((const void*)fcp::dq_kernel<64>, fcp::DqCfg<64>::LDS_BYTES, lds_done)) != FCP_OK) return rc;
    hipLaunchKernelGGL(fcp::dq_kernel<64>, grid_for(dq_units, 1), dim3(512), fcp::DqCfg<64>::LDS_BYTES, st, p, head_pair);
  }
  FCP_HIP_CHECK(hipGetLastError());
  return FCP_OK;
}

extern "C" int fcp_attn_bwd_step(const void* q, const void* k, const void* v, const void* d_o, const float* lse,
                                 const float* delta, const int32_t* cu_seqlens_kv, int32_t n_seqs,
                                 const fcp_work_desc* work, int64_t n_work, int32_t tq, int32_t tkv, int32_t hq,
                                 int32_t hkv, int32_t head_dim, float softmax_scale, float* dq_acc, float* dk_acc,
                                 float* dv_acc, void* scratch, size_t scratch_bytes, void* stream) {
  return bwd_step(q, k, v, d_o, lse, delta, cu_seqlens_kv, n_seqs, work, n_work, tq, tkv, hq, hkv, head_dim,
                  softmax_scale, nullptr, nullptr, dq_acc, dk_acc, dv_acc, scratch, scratch_bytes, stream);
}

extern "C" int fcp_attn_bwd_step_mixed(const void* q, const void* k, const void* v, const void* d_o, const float* lse,
                                       const float* delta, const int32_t* cu_seqlens_kv, int32_t n_seqs,
                                       const fcp_work_desc* work, int64_t n_work, int32_t tq, int32_t tkv, int32_t hq,
                                       int32_t hkv, int32_t head_dim, float softmax_scale, const int32_t* q_limit,
                                       const int32_t* k_from, float* dq_acc, float* dk_acc, float* dv_acc,
                                       void* scratch, size_t scratch_bytes, void* stream) {
  if (!q_limit || !k_from) {
    fcp::clear_error();
    return fail(FCP_ERR_INVALID_ARG, "fcp_attn_bwd_step_mixed: q_limit or k_from is NULL");
  }
  return bwd_step(q, k, v, d_o, lse, delta, cu_seqlens_kv, n_seqs, work, n_work, tq, tkv, hq, hkv, head_dim,
                  softmax_scale, q_limit, k_from, dq_acc, dk_acc, dv_acc, scratch, scratch_bytes, stream);
}

extern "C" int fcp_attn_bwd_step_direct(const void* q, const void* k, const void* v, const void* d_o, const float* lse,
                                        const float* delta, const int32_t* cu_seqlens_kv, int32_t n_seqs,
                                        const fcp_work_desc* work, int64_t n_work, int32_t tq, int32_t tkv, int32_t hq,
                                        int32_t hkv, int32_t head_dim, float softmax_scale, const int32_t* q_limit,
                                        const int32_t* k_from, float* dq_acc, float* dk_acc, float* dv_acc, void* dq_out,
                                        void* dk_out, void* dv_out, void* scratch, size_t scratch_bytes, void* stream) {
  fcp::clear_error();
  if (!dq_out || !dk_out || !dv_out) return fail(FCP_ERR_INVALID_ARG, "fcp_attn_bwd_step_direct: output pointer is NULL");
  if ((q_limit == nullptr) != (k_from == nullptr))
    return fail(FCP_ERR_INVALID_ARG, "fcp_attn_bwd_step_direct: q_limit and k_from go together");
  if ((reinterpret_cast<uintptr_t>(dq_out) | reinterpret_cast<uintptr_t>(dk_out) | reinterpret_cast<uintptr_t>(dv_out)) & 15u)
    return fail(FCP_ERR_INVALID_ARG, "fcp_attn_bwd_step_direct: outputs must be 16-byte aligned");
  return bwd_step(q, k, v, d_o, lse, delta, cu_seqlens_kv, n_seqs, work, n_work, tq, tkv, hq, hkv, head_dim,
                  softmax_scale, q_limit, k_from, dq_acc, dk_acc, dv_acc, scratch, scratch_bytes, stream, dq_out, dk_out,
                  dv_out);
}
