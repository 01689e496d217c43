// fcp_attn_fwd_step: partial causal attention of one CP rank for its ring steps.
//
// Function computed: softmax(scale Q K^T) V (paper Eq. 1, Sec. 3.1) with the causal mask
// (Sec. 4.3), restricted to the keys one ring step brings (ring-style CP, Sec. 3.2), for
// packed sequences of heterogeneous length (Sec. 4.1).  Per row the kernel emits the
// locally normalised output and LSE = ln sum exp(scaled scores).
//
// gfx950 design
//   * persistent 512-thread blocks (8 wave64, one block per CU, two waves per SIMD) pull
//     (query tile, head) units from per-XCD counters; the tile list is sorted longest-first by
//     the scheduler kernel;
//   * a unit = 128 query rows of one work item for two query heads that share a KV head (waves 0..3 take the
//     first head, waves 4..7 the second), or, when the heads per KV head are odd, 256 query rows for one
//     head; either way the eight waves share every K/V tile, each owns 32 rows and keeps its Q fragments
//     in registers for the whole unit;
//   * K and V stream through LDS in 64-key tiles filled by LDS-direct buffer loads (no register
//     staging), four stages, chunk-permuted so that row reads (K) and transpose reads (V)
//     run at the full LDS rate;
//   * scores are computed TRANSPOSED, S^T = K Q^T with v_mfma_f32_32x32x16_bf16: a lane then
//     holds 16 keys of ONE query column, so the row maximum and sum are in-lane reductions
//     plus a single exchange with the lane 32 away, and the exponentiated scores are already
//     in the A-operand layout of the second contraction O += P V, whose accumulator is then
//     [query x channel] with the channel on the lane; the epilogue stages the wave's tile in LDS and stores whole rows;
//   * PING-PONG: waves w and w+4 share a SIMD (measured).  Matrix and vector instructions of
//     DIFFERENT waves of a SIMD execute together almost perfectly, those of one wave hardly do.
//     Each wave therefore alternates a matrix slot (scores of tile t, O += P V of tile t-1)
//     with a vector slot (fills of tile t+2, then mask, maximum, exponentials, sum, conversion of tile t), and
//     waves 4..7 run one slot behind waves 0..3; a block barrier at every slot boundary keeps the two
//     halves in opposite slots, so a SIMD's matrix pipe is busy in every slot.  A slot lasts as long as the matrix
//     slot of the waves that are in it: nothing but the matrix instructions and their LDS reads is on that path;
//   * direct mode: a tile whose rows no other work item of the launch covers stores its normalised O as bf16 and
//     its LSE in their final places instead of a partial result;
//   * key tiles completely below the diagonal skip the mask; key tiles completely above a
//     wave's rows are not computed by that wave (it only keeps the barriers).

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
  const int32_t* q_limit;   // [tq] last key position each local query row sees, NULL = its own position (causal)
  uint16_t* o_out;          // running and direct mode: final O as bf16 [tq,hq,D], or NULL
  float* lse_out;           // direct mode: final LSE [hq,tq]
  int32_t running;          // 1: slot 0 of o_part / lse_part is the caller's running result, continued and rewritten
  int32_t direct;           // 1: a tile whose rows no other item of the launch covers writes o_out / lse_out, no partial
  int32_t tq, hq, hkv;
  int32_t head_pair;  // 1: a unit is a 128-row tile for TWO heads of one KV head; 0: a 256-row tile for one head
  float scale_log2;   // softmax_scale * log2(e)
};

constexpr float kRescaleThreshold = 8.f;   // log2 units
constexpr int kFwdAhead = 4;               // LDS fragments requested this many MFMAs before their use (3 and 6 measured: no better)

template <int D>
struct FwdCfg {
  static constexpr int BM = kFwdBM;               // 256 query rows per unit (32 per wave)
  static constexpr int BN = kFwdBN;               // 64 keys per LDS tile
  static constexpr int NWAVE = 8;
  using KT = RowTile<D>;
  using VT = TrTile<D>;
  static constexpr int KBYTES = KT::bytes(BN);
  static constexpr int VBYTES = VT::bytes(BN);
  static constexpr int NSTAGE = 4;                // LDS stages of one K and one V tile
  static constexpr int STAGE = KBYTES + VBYTES;
  static constexpr int LDS_BYTES = NSTAGE * STAGE;
  static constexpr int RPW = BN / NWAVE;          // tile rows each wave fills
  static constexpr int IPT = RPW / KT::RPI;       // fill instructions per wave per tile and tensor
  static constexpr int FILLS = 2 * IPT;           // ... per tile
  static constexpr int NKA = D == 128 ? 2 : 4;    // distinct per-lane K read addresses
  static constexpr int NVA = D / 32;              // distinct per-lane V^T read addresses
  static constexpr int NS = D / 16;               // MFMAs of one 32 x 32 score block
  static constexpr int KB_STRIDE = KT::row_base(32);
  static_assert(RPW % KT::RPI == 0 && FILLS < 16, "fill split");
};


template <int D>
__global__ __launch_bounds__(512, 1) void fwd_kernel(const FwdParams p) {
  using C = FwdCfg<D>;
  using KT = typename C::KT;
  using VT = typename C::VT;
  extern __shared__ __attribute__((aligned(256))) unsigned char smem[];
  __shared__ int32_t s_next_unit;
  __shared__ int32_t s_rec[16];
  __shared__ __attribute__((aligned(16))) float s_rowf[8][32];   // per wave: one factor per query row, see scale_rows()

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int grp = wave >> 2;                      // 0: waves 0..3, 1: waves 4..7 (one slot behind)
  const int l32 = lane & 31, g2 = lane >> 5;
  const int G = p.hq / p.hkv;
  const uint32_t lds0 = lds_offset(smem);

  // unit numbering: when the heads split evenly each XCD owns a contiguous eighth of them (so the K/V of a
  // KV head stay in one L2); a unit covers one head or, in head-pair mode, two consecutive heads
  const int hpu = p.head_pair ? 2 : 1;
  const bool per_xcd = (p.hq % (kNumXcd * hpu)) == 0;
  const int xcd = per_xcd ? (int)(blockIdx.x % kNumXcd) : 0;
  const int heads_here = per_xcd ? p.hq / kNumXcd : p.hq;
  const int units_per_tile = heads_here / hpu;
  UnitQueue uq;
  uq.init(p.hdr, p.tiles, xcd, units_per_tile, &s_next_unit, s_rec);

  // ---- per-lane constants -----------------------------------------------------------------
  const int kv_row_bytes = p.hkv * D * 2;
  // LDS-direct fills: the lane's global offset inside a tile (K and V are permuted differently);
  // instruction i of a wave adds i * RPI rows through the scalar offset (the permutations do not depend on i)
  const int kfill = fill_voff<KT>(C::RPW, wave, 0, lane, kv_row_bytes);
  const int vfill = fill_voff<VT>(C::RPW, wave, 0, lane, kv_row_bytes);
  // K row fragments (A operand of S^T = K Q^T): lane reads tile row l32 (+32 per key block), chunk 2 ks + g2
  int kaddr[C::NKA];
#pragma unroll
  for (int j = 0; j < C::NKA; ++j) kaddr[j] = tile_off<KT>(l32, 2 * j + g2);
  // V^T fragments (B operand of O += P V, columns d = 32 db + l32; k-slots = keys 16 tt + {4 g2 + [0,4),
  // 8 + 4 g2 + [0,4)}).  Transpose read: inside a 16-lane block lane i supplies the address of key row
  // (i / 4), channels 4 (i % 4) + [0,4); block b covers channels 16 (b % 2) + [0,16) for key group b / 2.
  int vaddr[C::NVA];
  {
    const int row0 = 4 * g2 + ((lane & 15) >> 2);
    const int chunk0 = 2 * ((lane >> 4) & 1) + ((lane & 3) >> 1);
#pragma unroll
    for (int db = 0; db < C::NVA; ++db) vaddr[db] = C::KBYTES + tile_off<VT>(row0, 4 * db + chunk0) + 8 * (lane & 1);
  }
  for (;;) {
    const int unit = uq.current(&s_next_unit);
    if (unit >= uq.n_units) break;
    const QTile t = read_record<QTile, 12>(s_rec);
    const int head = xcd * heads_here + (unit % units_per_tile) * hpu + (p.head_pair ? grp : 0);
    const int kvh = head / G;

    const int wave_r0 = (p.head_pair ? (wave & 3) : wave) * 32;
    const bool wave_active = wave_r0 < t.rows;
    const int my_row = wave_r0 + l32;
    const bool row_valid = my_row < t.rows;
    const int row_ld = min(my_row, t.rows - 1);
    // Last key position the lane's row sees, and the least and greatest such limit among the wave's rows (the limits
    // grow with the row): the rows' own positions under the causal mask, else the caller's table.
    int q_lim = t.q_pos0 + my_row;
    int wave_first_lim = t.q_pos0 + wave_r0;
    int wave_last_lim = t.q_pos0 + min(wave_r0 + 31, t.rows - 1);
    if (p.q_limit) {
      const int32_t* ql = p.q_limit + t.q_row0;
      q_lim = ql[row_ld];
      wave_first_lim = ql[min(wave_r0, t.rows - 1)];
      wave_last_lim = ql[min(wave_r0 + 31, t.rows - 1)];
      __builtin_amdgcn_s_waitcnt(kWaitVm0);   // before any fill is in flight: later waits count the fills only
    }

    // Key tiles of the unit: nt0 of segment 0, then nt1 of segment 1 (64 keys each, the last of a segment
    // may be ragged).  A wave computes a prefix of them: the tiles its last row sees.
    const int nt0 = (t.vis[0] + C::BN - 1) / C::BN, nt1 = (t.vis[1] + C::BN - 1) / C::BN;
    const int n_iter = nt0 + nt1;
    int n_w = 0;
    if (wave_active) {
      const int v0 = max(0, min(t.vis[0], wave_last_lim - t.k_pos0[0] + 1));
      const int v1 = max(0, min(t.vis[1], wave_last_lim - t.k_pos0[1] + 1));
      const int w0 = (v0 + C::BN - 1) / C::BN, w1 = (v1 + C::BN - 1) / C::BN;
      n_w = w0 == nt0 ? w0 + w1 : w0;
    }
    // A buffer resource per segment whose extent ends with the last visible key, so rows past it
    // arrive as zeros.
    i32x4 rk[2], rv[2];
#pragma unroll
    for (int s = 0; s < 2; ++s) {
      const int64_t off = ((int64_t)t.kv_row0[s] * p.hkv + kvh) * D;
      const int bytes = t.vis[s] > 0 ? (t.vis[s] - 1) * kv_row_bytes + D * 2 : 0;
      rk[s] = buffer_rsrc(p.k + off, bytes);
      rv[s] = buffer_rsrc(p.v + off, bytes);
    }
    // This wave's share (RPW rows of K and of V, FILLS instructions) of the LDS-direct fill of the NEXT tile in
    // list order into the next stage (tiles are filled strictly in order 0, 1, 2, ...).  A prologue fill past the end of
    // a one-tile list lies outside the resource's range, loads nothing and writes zeros; the loop issues none.  The running
    // state keeps the scalar work per call small.
    i32x4 f_rk = rk[0], f_rv = rv[0];
    int f_left = nt0;                      // tiles left in segment 0 while it is being filled
    bool f_seg0 = true;
    int f_soff = 0;                        // byte offset of the next tile in its segment
    uint32_t f_dst = lds0 + KT::row_base(C::RPW * wave);   // this wave's rows in the next stage
    const uint32_t f_dst_end = lds0 + C::NSTAGE * C::STAGE;
    static_assert(KT::row_base(C::RPW * 7 + KT::RPI) == KT::row_base(C::RPW * 7) + KT::row_base(KT::RPI),
                  "a wave's rows start on a padding group boundary");
    const uint32_t f_vdelta = C::KBYTES + VT::row_base(C::RPW * wave) - KT::row_base(C::RPW * wave);
    auto fill_next = [&]() {
      if (f_seg0 && f_left == 0) { f_rk = rk[1]; f_rv = rv[1]; f_seg0 = false; f_soff = 0; }   // past segment 1: out of range
#pragma unroll
      for (int i = 0; i < C::IPT; ++i) {
        lds_fill_b128(f_rk, f_dst + KT::row_base(KT::RPI * i), kfill, f_soff + i * KT::RPI * kv_row_bytes);
        lds_fill_b128(f_rv, f_dst + f_vdelta + VT::row_base(VT::RPI * i), vfill, f_soff + i * VT::RPI * kv_row_bytes);
      }
      --f_left;
      f_soff += C::BN * kv_row_bytes;
      f_dst += C::STAGE;
      if (f_dst >= f_dst_end) f_dst -= C::NSTAGE * C::STAGE;
    };

    bf16x8 qf[D / 16];
    int s_q_area = 0;
    // Prologue fills: tile 0, the wave's Q rows, tile 1 - in the order they are needed: the first slot starts when
    // all but tile 1 have landed.  The previous unit's last barrier guarantees that no wave still reads the stages.
    fill_next();

    // Q fragments: B operand of S^T = K Q^T.  Lane holds column q = l32, channels 16 ks + 8 g2 + [0,8).  Loaded in
    // that form from global memory an instruction would touch 32 cache lines for 32 bytes of each; instead the wave's
    // 32 rows come in whole (LDS-direct fills of RPI rows each) beside the first two key tiles, into the part of stages
    // 2 and 3 that is the wave's own until the first slot's barrier, and the fragments are read from there.  Rows past
    // the tile's last arrive as zeros.
    {
      using QT = DualTile<D>;
      static_assert(C::NWAVE * QT::bytes(32) <= 2 * C::STAGE, "the waves' Q tiles fit into two stages");
      int lane_p = lane;                            // addresses formed here, not ahead of the unit loop (registers)
      asm volatile("" : "+v"(lane_p));
      const int q_row_bytes = p.hq * D * 2;
      const int n_wave_rows = t.rows - wave_r0;
      const i32x4 rq = buffer_rsrc(p.q + ((int64_t)(t.q_row0 + wave_r0) * p.hq + head) * D,
                                   n_wave_rows > 0 ? (min(n_wave_rows, 32) - 1) * q_row_bytes + D * 2 : 0);
      const int area = 2 * C::STAGE + wave * QT::bytes(32);
#pragma unroll
      for (int i = 0; i < 32 / QT::RPI; ++i)
        lds_fill_b128(rq, lds0 + area + QT::row_base(QT::RPI * i), fill_voff<QT>(32, 0, i, lane_p, q_row_bytes), 0);
      s_q_area = area;
    }
    fill_next();
    f32x16 oacc[D / 32];
#pragma unroll
    for (int db = 0; db < D / 32; ++db) oacc[db] = zero16();
    float m_run = -INFINITY;   // running maximum in log2 units (score * scale_log2)
    float l_run = 0.f;         // this lane's share of the running sum
    const int slot = p.running ? 0 : t.step;
    if (p.running) {
      // The caller's merged result of the earlier ring steps is one more block of keys already folded into the
      // state: maximum = its LSE, sum 1 (held by the lower half-wave), accumulator = its normalised O.  A row
      // without earlier keys (LSE = -inf) starts like any other.
      const float lse_prev = p.lse_part[(int64_t)head * p.tq + t.q_row0 + row_ld];
      const int row_bytes = p.hq * D * 4;
      const int n_wave_rows = t.rows - wave_r0;
      const __amdgpu_buffer_rsrc_t ri = __builtin_amdgcn_make_buffer_rsrc(
          (void*)(p.o_part + ((int64_t)(t.q_row0 + wave_r0) * p.hq + head) * D), (short)0,
          n_wave_rows > 0 ? (n_wave_rows - 1) * row_bytes + D * 4 : 0, 0x00020000);
      const int o_voff = 4 * g2 * row_bytes + 4 * l32;
#pragma unroll
      for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i)
          oacc[db][i] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(
              ri, o_voff, (8 * (i / 4) + (i % 4)) * row_bytes + 128 * db, 0));
      const bool has_prev = lse_prev > -INFINITY;
      if (has_prev) {
        m_run = lse_prev * kLog2e;
        l_run = g2 == 0 ? 1.f : 0.f;
      }
      __builtin_amdgcn_s_waitcnt(kWaitVm0);   // not inside the tile loop, where a wait would also cover the fills
      // whatever o_run holds for a row without earlier keys is dropped (the flag travels like a row factor)
      s_rowf[wave][l32] = has_prev ? 1.f : 0.f;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const f32x4 a = *reinterpret_cast<const f32x4*>(&s_rowf[wave][8 * j + 4 * g2]);
#pragma unroll
        for (int db = 0; db < D / 32; ++db)
#pragma unroll
          for (int e = 0; e < 4; ++e) oacc[db][4 * j + e] = a[e] != 0.f ? oacc[db][4 * j + e] : 0.f;
      }
    }
    f32x16 sacc[2];            // scores of the current tile: sacc[kb][i] = key 32 kb + 8 (i/4) + 4 g2 + (i%4), query l32
    bf16x8 pf[4];              // P^T of the current tile as B operands: k-step tt covers keys 16 tt .. 16 tt + 15

    // ---- the two slots ------------------------------------------------------------------------
    // K row fragment f of a tile: key block f / NS, channels 16 (f % NS) + 8 g2 + [0,8)
    auto k_frag = [&](const int (&ka)[C::NKA], int f) -> bf16x8 {
      const int kb = f / C::NS, ks = f % C::NS;
      return *reinterpret_cast<const bf16x8*>(smem + ka[ks % C::NKA] + (ks / C::NKA) * (C::NKA * 32) + kb * C::KB_STRIDE);
    };
    // V^T fragment g: keys 16 (g / NVA) + .., channels 32 (g % NVA) + l32
    auto v_frag = [&](const int (&va)[C::NVA], int g) -> bf16x8 {
      const int tt = g / C::NVA, db = g % C::NVA;
      return tr_read_8(smem + va[db] + tt * (16 * VT::row_base(1)), 8 * VT::row_base(1));
    };
    // Matrix slot of step `it`: scores of tile it (score_part), O += P V of tile it - 1 (pv_part), each present ONCE in
    // the program and run or skipped as a whole.  (Variants of the slot that repeat the second contraction on several
    // paths make the register allocator keep two copies of the O accumulator and move 64 registers between them in
    // every step.)  The order inside a part is written out MFMA by MFMA and fenced so that every LDS fragment is
    // requested kAhead MFMAs before the one that consumes it; the first fragments of the second contraction are
    // requested before the scores (pv_head), so that it starts without waiting for LDS.
    constexpr int kAhead = kFwdAhead;
    bf16x8 vhead[kAhead];
    auto pv_head = [&](int it) {
      int va[C::NVA];
      const int voff = ((it - 1) & (C::NSTAGE - 1)) * C::STAGE;
#pragma unroll
      for (int db = 0; db < C::NVA; ++db) va[db] = vaddr[db] + voff;
#pragma unroll
      for (int x = 0; x < kAhead; ++x) vhead[x] = v_frag(va, x);
    };
    auto score_part = [&](int it) {
      constexpr int N = 2 * C::NS;
      int ka[C::NKA];
      const int koff = (it & (C::NSTAGE - 1)) * C::STAGE;
#pragma unroll
      for (int j = 0; j < C::NKA; ++j) ka[j] = kaddr[j] + koff;
      bf16x8 fr[N];
      auto request = [&](int x) { if (x < N) fr[x] = k_frag(ka, x); };
#pragma unroll
      for (int x = 0; x < kAhead; ++x) request(x);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int x = 0; x < N; ++x) {
        sacc[x / C::NS] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[x], qf[x % C::NS], x % C::NS == 0 ? zero16() : sacc[x / C::NS], 0, 0, 0);
        request(x + kAhead);
        __builtin_amdgcn_sched_barrier(0);
      }
    };
    auto pv_part = [&](int it) {
      constexpr int N = 4 * C::NVA;
      static_assert(kAhead <= N, "the head fragments are all used");
      int va[C::NVA];
      const int voff = ((it - 1) & (C::NSTAGE - 1)) * C::STAGE;
#pragma unroll
      for (int db = 0; db < C::NVA; ++db) va[db] = vaddr[db] + voff;
      bf16x8 fr[N];
#pragma unroll
      for (int x = 0; x < kAhead; ++x) fr[x] = vhead[x];
      auto request = [&](int x) { if (x < N) fr[x] = v_frag(va, x); };
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int x = 0; x < N; ++x) {
        oacc[x % C::NVA] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pf[x / C::NVA], fr[x], oacc[x % C::NVA], 0, 0, 0);
        request(x + kAhead);
        __builtin_amdgcn_sched_barrier(0);
      }
    };
    auto tile_geom = [&](int it, int& k_pos0, int& n_valid) {
      const int s = it >= nt0 ? 1 : 0;
      const int kt = it - (s ? nt0 : 0);
      k_pos0 = t.k_pos0[s] + kt * C::BN;
      n_valid = min(C::BN, t.vis[s] - kt * C::BN);
    };
    // Vector slot of step `it`: mask, running maximum (lazy: raised only when some row of the wave outgrows it
    // by 2^kRescaleThreshold, until then probabilities may exceed 1 by at most that factor), exponentials, row
    // sum, conversion to bf16.  The row sum is taken over the unrounded fp32 values (summing the bf16-rounded
    // ones would cost up to 2^-9 relative on a peaked row, more than the 1e-3 the LSE has to hold).
    // O is accumulated as [query x channel] with the channel on the lane (register i = row 8 (i/4) + 4 g2 + i%4 of the
    // wave's 32), so that the epilogue stores whole 128-byte lines; the row statistics live one row per lane.  A
    // per-row factor therefore goes through the wave's LDS slot: every lane leaves its row's factor, then picks up
    // the four factors of each of its register groups.  (Rare: the rescale is lazy.)
    auto scale_rows = [&](float f) {
      s_rowf[wave][l32] = f;                       // both half-waves hold the same value for a row
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const f32x4 a = *reinterpret_cast<const f32x4*>(&s_rowf[wave][8 * j + 4 * g2]);
#pragma unroll
        for (int db = 0; db < D / 32; ++db)
#pragma unroll
          for (int e = 0; e < 4; ++e) oacc[db][4 * j + e] *= a[e];
      }
    };
    auto vector_slot = [&](int it) {
      int k_pos0, n_valid;
      tile_geom(it, k_pos0, n_valid);
      if ((k_pos0 + C::BN - 1 > wave_first_lim) || (n_valid < C::BN)) {   // wave-uniform: mask edge / segment end
        const int lim = min(n_valid, q_lim - k_pos0 + 1) - 4 * g2;        // key index (minus 4 g2) below which the lane sees
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int i = 0; i < 16; ++i)
            if (32 * kb + 8 * (i / 4) + (i % 4) >= lim) sacc[kb][i] = -INFINITY;
      }
      float mx = max3(sacc[0][0], sacc[0][1], sacc[1][0]);
      mx = fmaxf(mx, sacc[1][1]);
#pragma unroll
      for (int i = 2; i < 16; i += 2) mx = max3(max3(mx, sacc[0][i], sacc[0][i + 1]), sacc[1][i], sacc[1][i + 1]);
      mx = lane32_partner_max(mx) * p.scale_log2;
      if (__builtin_amdgcn_ballot_w64(mx > m_run + kRescaleThreshold) != 0) {
        const float m_new = fmaxf(m_run, mx);
        const float alpha = __builtin_amdgcn_exp2f(m_run - (m_new == -INFINITY ? 0.f : m_new));
        m_run = m_new;
        l_run *= alpha;
        scale_rows(alpha);
      }
      const float m_use = m_run == -INFINITY ? 0.f : m_run;
      float psum = 0.f;
#pragma unroll
      for (int e = 0; e < 32; e += 2) {
        const float e0 = __builtin_amdgcn_exp2f(fmaf(sacc[e / 16][e % 16], p.scale_log2, -m_use));
        const float e1 = __builtin_amdgcn_exp2f(fmaf(sacc[e / 16][e % 16 + 1], p.scale_log2, -m_use));
        psum += e0;
        psum += e1;
        pf[e / 8][e % 8] = (__bf16)e0;
        pf[e / 8][e % 8 + 1] = (__bf16)e1;
      }
      l_run += psum;
    };

    // ---- the unit -------------------------------------------------------------------------------
    // Step `it` of a wave = matrix slot (scores of tile it; second contraction of tile it-1) then vector slot (fills
    // of tile it+2; softmax of tile it).  Waves 4..7 start one slot late.  The fills go out at the start of the
    // VECTOR slot: the matrix slot is the longer one and every slot lasts as long as the matrix slot of the four waves
    // that are in it, so nothing else belongs on its path (measured: -2.5 %).  A fill overwrites stage (it+2) % 4,
    // whose previous tile it-2 was last read in matrix slot it-1 of both halves, two and one slots earlier; a wave
    // waits for it at the end of its matrix slot it+1, and tile it+2 is first read in matrix slot it+2 of the early
    // waves, which starts after the late waves' matrix slot it+1 has ended with the same wait.
    __builtin_amdgcn_s_waitcnt(kWaitVm0 | C::FILLS);   // everything but this wave's part of tile 1 (the newest loads)
    {
      using QT = DualTile<D>;
      int lane_p = lane;
      asm volatile("" : "+v"(lane_p));
#pragma unroll
      for (int ks = 0; ks < D / 16; ++ks)
        qf[ks] = *reinterpret_cast<const bf16x8*>(smem + s_q_area + tile_off<QT>(lane_p & 31, 2 * ks + (lane_p >> 5)));
      __builtin_amdgcn_s_waitcnt(0xC07F);           // lgkmcnt(0): in registers before anybody fills stage 2
    }
    __syncthreads();                       // tile 0 has landed (tile 1: by the first slot boundary)
    if (grp == 1) __syncthreads();
    for (int it = 0; it <= n_iter; ++it) {
      const bool do_s = it < n_w, do_pv = it > 0 && it - 1 < n_w;
      // the matrix stream goes first at the SIMD's issue port: an MFMA is wanted every 32 cycles and must not
      // queue behind the partner wave's vector instructions
      __builtin_amdgcn_s_setprio(3);
      if (do_pv) pv_head(it);
      if (do_s) score_part(it);
      if (do_pv) pv_part(it);
      __builtin_amdgcn_s_setprio(0);
      // slot boundary: this wave's fills (issued a step ago) have landed, then everybody meets
      __builtin_amdgcn_s_waitcnt(kWaitVm0);
      __syncthreads();
      if (it + 2 < n_iter) fill_next();      // (nothing in flight when the loop ends: the epilogue reuses the stages)
      if (do_s) vector_slot(it);
      __syncthreads();
    }
    if (grp == 0) __syncthreads();

    // The next unit's record and the number of the unit after it start their trips here, ahead of the epilogue's
    // stores (waiting for them later must not mean waiting for those stores).
    uq.prefetch();
    // ---- epilogue: normalise, write partial O (fp32) and LSE --------------------------------
    const float l_tot = lane32_partner_sum(l_run);
    const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
    scale_rows(inv);
    // Direct mode: the tile's rows get all their keys in this unit, so the normalised O is the final one.
    const bool direct = p.direct && (t.flags & kFlagQExclusive) != 0;
    // The tile leaves as whole rows through the wave's staging area (the stages are free: every wave has passed its
    // last matrix slot and no fill is in flight); the rows are reached through a buffer resource that ends with the
    // tile's last row, so that stores past it are dropped.
    using OUT = RowStage<D>;
    static_assert(C::NWAVE * OUT::BYTES <= C::LDS_BYTES, "staging areas inside the stages");
    unsigned char* const obuf = smem + wave * OUT::BYTES;
    int lane_e = lane;                              // see RowStage::flush
    asm volatile("" : "+v"(lane_e));
    const int l32e = lane_e & 31, g2e = lane_e >> 5;
    const int n_wave_rows = t.rows - wave_r0;
    if (!direct) {                                  // partial O, fp32: D / 2 channels per pass
      const int row_bytes = p.hq * D * 4;
      const __amdgpu_buffer_rsrc_t ro = __builtin_amdgcn_make_buffer_rsrc(
          (void*)(p.o_part + (int64_t)slot * ((int64_t)p.tq * p.hq * D) + ((int64_t)(t.q_row0 + wave_r0) * p.hq + head) * D),
          (short)0, n_wave_rows > 0 ? (n_wave_rows - 1) * row_bytes + D * 4 : 0, 0x00020000);
#pragma unroll
      for (int h = 0; h < 2; ++h) {
#pragma unroll
        for (int db = 0; db < D / 64; ++db)
#pragma unroll
          for (int i = 0; i < 16; ++i)
            OUT::put_f32(obuf, OUT::reg_row(i, g2e), 32 * db + l32e, oacc[h * (D / 64) + db][i]);
        OUT::flush(obuf, lane_e, ro, row_bytes, h * D * 2);
      }
    }
    if (p.o_out && (p.running || direct)) {   // the final rows as bf16
      const int row_bytes = p.hq * D * 2;
      const __amdgpu_buffer_rsrc_t rb = __builtin_amdgcn_make_buffer_rsrc(
          (void*)(p.o_out + ((int64_t)(t.q_row0 + wave_r0) * p.hq + head) * D), (short)0,
          n_wave_rows > 0 ? (n_wave_rows - 1) * row_bytes + D * 2 : 0, 0x00020000);
#pragma unroll
      for (int db = 0; db < D / 32; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) OUT::put_bf16(obuf, OUT::reg_row(i, g2e), 32 * db + l32e, oacc[db][i]);
      OUT::flush(obuf, lane_e, rb, row_bytes, 0);
    }
    if (row_valid && g2 == 0) {
      const float lse = l_tot > 0.f ? (m_run + __builtin_amdgcn_logf(l_tot)) * kLn2 : -INFINITY;
      float* dst = direct ? p.lse_out : p.lse_part + (int64_t)slot * ((int64_t)p.hq * p.tq);
      dst[(int64_t)head * p.tq + t.q_row0 + my_row] = lse;
    }
    uq.advance(&s_next_unit, s_rec);   // hand the next unit to the block (barrier: LDS stages are free)
  }
}

}  // namespace
}  // namespace fcp

using fcp::fail;

// Both entry points; q_limit == NULL is the causal mask.
static int fwd_step(const void* q, const void* k, const void* v, const int32_t* cu_seqlens_kv,
                    int32_t n_seqs, const fcp_work_desc* work, int64_t n_work, int32_t n_parts,
                    int32_t tq, int32_t tkv, int32_t hq, int32_t hkv, int32_t head_dim,
                    float softmax_scale, const int32_t* q_limit, float* o_part, float* lse_part, void* scratch,
                    size_t scratch_bytes, void* stream, bool running = false, void* o_out = nullptr,
                    float* lse_out = nullptr) {
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
  if (reinterpret_cast<uintptr_t>(scratch) & 255u) return fail(FCP_ERR_INVALID_ARG, "fcp_attn_fwd_step: scratch must be 256-byte aligned");
  const size_t need = fcp_scratch_bytes(FCP_SCRATCH_FWD, tq, tkv, hq, hkv, head_dim, n_work, n_parts);
  if (scratch_bytes < need) return fail(FCP_ERR_CAPACITY, "fcp_attn_fwd_step: scratch %zu < %zu bytes", scratch_bytes, need);
  if ((int64_t)tq * hq * head_dim * (int64_t)n_parts > ((int64_t)1 << 40))
    return fail(FCP_ERR_UNSUPPORTED, "fcp_attn_fwd_step: partial output too large");

  hipStream_t st = (hipStream_t)stream;
  const int64_t cap = fcp::q_tile_cap(tq, tkv, n_work, n_parts);
  if (cap > INT32_MAX / 64) return fail(FCP_ERR_UNSUPPORTED, "fcp_attn_fwd_step: too many tiles");
  // two heads of one KV head per unit when the heads pair up, else twice the rows for one head
  const int head_pair = ((hq / hkv) % 2 == 0) ? 1 : 0;
  const bool direct = lse_out != nullptr;
  // direct mode: which rows get their final result from one unit and which are merged from partials is worked out on
  // extra blocks of the scheduling launch
  fcp::RowStates rs{};
  if (direct) {
    rs.q_state = fcp::fwd_q_state(scratch, n_work, tq, tkv, n_parts);
    rs.q_row_elems = hq * head_dim; rs.kv_row_elems = hkv * head_dim;
    rs.n_parts = n_parts; rs.check_step = true;
  }
  int rc = fcp::launch_schedule(false, head_pair ? fcp::kFwdBM / 2 : fcp::kFwdBM, fcp::kFwdBN, (int64_t)hkv * head_dim * 2, q_limit, nullptr, work, n_work, cu_seqlens_kv, n_seqs, tq, tkv, n_parts, cap, scratch,
                                running ? nullptr : lse_part, (int64_t)n_parts * hq * tq, st, direct ? &rs : nullptr);
  if (rc != FCP_OK) return rc;
  if (tq == 0 || n_work == 0) return FCP_OK;

  fcp::FwdParams p;
  p.q = (const uint16_t*)q; p.k = (const uint16_t*)k; p.v = (const uint16_t*)v;
  p.hdr = (fcp::SchedHeader*)scratch;
  p.tiles = fcp::sched_tiles(scratch, n_work);
  p.o_part = o_part; p.lse_part = lse_part;
  p.q_limit = q_limit;
  p.running = running ? 1 : 0;
  p.o_out = (uint16_t*)o_out;
  p.lse_out = lse_out;
  p.direct = direct ? 1 : 0;
  p.tq = tq; p.hq = hq; p.hkv = hkv;
  p.head_pair = head_pair;
  p.scale_log2 = softmax_scale * 1.4426950408889634f;

  int dev = 0, n_cu = 256;
  FCP_HIP_CHECK(hipGetDevice(&dev));
  FCP_HIP_CHECK(hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev));
  int64_t units = cap * (hq / (head_pair ? 2 : 1));
  int64_t blocks = n_cu;                               // one 512-thread block per CU
  if (blocks > units) blocks = (units + 7) / 8 * 8;   // keep a multiple of the XCD count
  if (blocks < 8) blocks = 8;
  static std::atomic<uint64_t> lds_done[2];
  if (head_dim == 128) {
    if ((rc = fcp::raise_lds_limit((const void*)fcp::fwd_kernel<128>, fcp::FwdCfg<128>::LDS_BYTES, lds_done[0])) != FCP_OK) return rc;
    hipLaunchKernelGGL(fcp::fwd_kernel<128>, dim3((unsigned)blocks), dim3(512), fcp::FwdCfg<128>::LDS_BYTES, st, p);
  } else {
    if ((rc = fcp::raise_lds_limit((const void*)fcp::fwd_kernel<64>, fcp::FwdCfg<64>::LDS_BYTES, lds_done[1])) != FCP_OK) return rc;
    hipLaunchKernelGGL(fcp::fwd_kernel<64>, dim3((unsigned)blocks), dim3(512), fcp::FwdCfg<64>::LDS_BYTES, st, p);
  }
  FCP_HIP_CHECK(hipGetLastError());
  return FCP_OK;
}

// ---- fcp_attn_fwd_step_static: the same call with the scheduler's work area in a static device array ----------
// For callers that cannot allocate device memory.  The array below exists once per GPU the library runs on, for
// the life of the process.  In host code its NAME is only a handle for the runtime: the device address comes from
// hipGetSymbolAddress (once per device, with that device current) and only that address is ever handed to a kernel.
static __device__ __align__(256) unsigned char fcp_static_scratch[FCP_STATIC_SCRATCH_BYTES];

static int static_scratch_address(void** out) {
  constexpr int kMaxDev = 64;
  static std::atomic<void*> addr[kMaxDev];       // zero-initialised; one slot per device ordinal
  int dev = 0;
  FCP_HIP_CHECK(hipGetDevice(&dev));
  void* p = (dev >= 0 && dev < kMaxDev) ? addr[dev].load(std::memory_order_acquire) : nullptr;
  if (!p) {
    FCP_HIP_CHECK(hipGetSymbolAddress(&p, HIP_SYMBOL(fcp_static_scratch)));
    if (!p) return fail(FCP_ERR_HIP, "fcp_attn_fwd_step_static: the static work area has no device address");
    if (dev >= 0 && dev < kMaxDev) addr[dev].store(p, std::memory_order_release);   // (two threads store the same value)
  }
  *out = p;
  return FCP_OK;
}

extern "C" int fcp_attn_fwd_step_static(const void* q, const void* k, const void* v, const int32_t* cu_seqlens_kv,
                                        int32_t n_seqs, const fcp_work_desc* work, int64_t n_work, int32_t n_parts,
                                        int32_t tq, int32_t tkv, int32_t hq, int32_t hkv, int32_t head_dim,
                                        float softmax_scale, float* o_part, float* lse_part, void* stream) {
  fcp::clear_error();
  if (tq < 0 || tkv < 1 || n_work < 0 || n_parts < 1 || hq < 1 || hkv < 1)
    return fail(FCP_ERR_INVALID_ARG, "fcp_attn_fwd_step_static: bad sizes");
  const size_t need = fcp_scratch_bytes(FCP_SCRATCH_FWD, tq, tkv, hq, hkv, head_dim, n_work, n_parts);
  if (need > (size_t)FCP_STATIC_SCRATCH_BYTES)
    return fail(FCP_ERR_CAPACITY, "fcp_attn_fwd_step_static: this call needs a work area of %zu bytes, the static one has %zu "
                                  "(use fcp_attn_fwd_step with a caller-owned scratch buffer)", need, (size_t)FCP_STATIC_SCRATCH_BYTES);
  void* area = nullptr;
  const int rc = static_scratch_address(&area);
  if (rc != FCP_OK) return rc;
  // every part of the area that the kernels read is written first by the scheduling launch of the same call (header,
  // counters, offsets, flags, tile records), so what the previous call left needs no clearing
  return fwd_step(q, k, v, cu_seqlens_kv, n_seqs, work, n_work, n_parts, tq, tkv, hq, hkv, head_dim, softmax_scale,
                  nullptr, o_part, lse_part, area, (size_t)FCP_STATIC_SCRATCH_BYTES, stream);
}

extern "C" int fcp_attn_fwd_step(const void* q, const void* k, const void* v, const int32_t* cu_seqlens_kv,
                                 int32_t n_seqs, const fcp_work_desc* work, int64_t n_work, int32_t n_parts,
                                 int32_t tq, int32_t tkv, int32_t hq, int32_t hkv, int32_t head_dim,
                                 float softmax_scale, float* o_part, float* lse_part, void* scratch,
                                 size_t scratch_bytes, void* stream) {
  return fwd_step(q, k, v, cu_seqlens_kv, n_seqs, work, n_work, n_parts, tq, tkv, hq, hkv, head_dim, softmax_scale,
                  nullptr, o_part, lse_part, scratch, scratch_bytes, stream);
}

extern "C" int fcp_attn_fwd_step_mixed(const void* q, const void* k, const void* v, const int32_t* cu_seqlens_kv,
                                       int32_t n_seqs, const fcp_work_desc* work, int64_t n_work, int32_t n_parts,
                                       int32_t tq, int32_t tkv, int32_t hq, int32_t hkv, int32_t head_dim,
                                       float softmax_scale, const int32_t* q_limit, float* o_part, float* lse_part,
                                       void* scratch, size_t scratch_bytes, void* stream) {
  if (!q_limit) { fcp::clear_error(); return fail(FCP_ERR_INVALID_ARG, "fcp_attn_fwd_step_mixed: q_limit is NULL"); }
  return fwd_step(q, k, v, cu_seqlens_kv, n_seqs, work, n_work, n_parts, tq, tkv, hq, hkv, head_dim, softmax_scale,
                  q_limit, o_part, lse_part, scratch, scratch_bytes, stream);
}

extern "C" int fcp_attn_fwd_step_running(const void* q, const void* k, const void* v, const int32_t* cu_seqlens_kv,
                                         int32_t n_seqs, const fcp_work_desc* work, int64_t n_work, int32_t tq,
                                         int32_t tkv, int32_t hq, int32_t hkv, int32_t head_dim, float softmax_scale,
                                         const int32_t* q_limit, float* o_run, float* lse_run, void* o_out,
                                         void* scratch, size_t scratch_bytes, void* stream) {
  if (o_out && (reinterpret_cast<uintptr_t>(o_out) & 3u)) {
    fcp::clear_error();
    return fail(FCP_ERR_INVALID_ARG, "fcp_attn_fwd_step_running: o_out must be 4-byte aligned");
  }
  return fwd_step(q, k, v, cu_seqlens_kv, n_seqs, work, n_work, 1, tq, tkv, hq, hkv, head_dim, softmax_scale, q_limit,
                  o_run, lse_run, scratch, scratch_bytes, stream, true, o_out);
}

extern "C" int fcp_attn_fwd_step_direct(const void* q, const void* k, const void* v, const int32_t* cu_seqlens_kv,
                                        int32_t n_seqs, const fcp_work_desc* work, int64_t n_work, int32_t n_parts,
                                        int32_t tq, int32_t tkv, int32_t hq, int32_t hkv, int32_t head_dim,
                                        float softmax_scale, const int32_t* q_limit, float* o_part, float* lse_part,
                                        void* o, float* lse, void* scratch, size_t scratch_bytes, void* stream) {
  if (!o || !lse || (reinterpret_cast<uintptr_t>(o) & 15u)) {
    fcp::clear_error();
    return fail(FCP_ERR_INVALID_ARG, "fcp_attn_fwd_step_direct: o / lse NULL or o not 16-byte aligned");
  }
  return fwd_step(q, k, v, cu_seqlens_kv, n_seqs, work, n_work, n_parts, tq, tkv, hq, hkv, head_dim, softmax_scale,
                  q_limit, o_part, lse_part, scratch, scratch_bytes, stream, false, o, lse);
}
