// Bandwidth-bound row kernels: log-sum-exp merge of the ring-step partials, the backward
// prologue delta = rowsum(dO * O), and the fp32 -> bf16 cast of the gradient accumulators.
//
// The paper computes attention (Eq. 1) ring-style over a CP group (Sec. 3.2); each ring
// step sees a different key set, so its softmax is normalised locally and the per-step
// results are combined exactly by weighting with exp(LSE_s - LSE).
#include "fcp_internal.h"

namespace fcp {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ inline uint32_t bf16_rne(float f) {           // one bf16 in the low 16 bits
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return 0x7fc0u;   // NaN
  return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}
__device__ inline uint32_t pack_bf16(float lo, float hi) { return bf16_rne(lo) | (bf16_rne(hi) << 16); }
__device__ inline float bf16_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ inline float bf16_hi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }

constexpr int kMaxParts = 16;   // partial slots held in registers by one merge thread

// Merge of one (row, head) by the D/8 threads that own it: thread c8 has 8 consecutive channels.
template <int D>
__device__ inline void merge_row_head(const float* __restrict__ o_part, const float* __restrict__ lse_part, int n_parts,
                                      int tq, int hq, uint32_t* __restrict__ o, float* __restrict__ lse, int row, int h,
                                      int c8) {
  const int64_t lse_stride = (int64_t)hq * tq;
  const int64_t o_stride = (int64_t)tq * hq * D;
  float ls[kMaxParts];
  float m = -INFINITY;
#pragma unroll
  for (int p = 0; p < kMaxParts; ++p) {
    ls[p] = p < n_parts ? lse_part[p * lse_stride + (int64_t)h * tq + row] : -INFINITY;
    m = fmaxf(m, ls[p]);
  }
  const float m_safe = m == -INFINITY ? 0.f : m;
  float tot = 0.f;
#pragma unroll
  for (int p = 0; p < kMaxParts; ++p) {
    ls[p] = __expf(ls[p] - m_safe);       // exp(-inf) = 0
    tot += ls[p];
  }
  const float inv = tot > 0.f ? 1.f / tot : 0.f;
  f32x4 a0 = {0, 0, 0, 0}, a1 = {0, 0, 0, 0};
  const int64_t off = ((int64_t)row * hq + h) * D + c8 * 8;
#pragma unroll
  for (int p = 0; p < kMaxParts; ++p) {
    if (p < n_parts && ls[p] > 0.f) {     // skipped slots are never read
      const f32x4* src = reinterpret_cast<const f32x4*>(o_part + p * o_stride + off);
      const float w = ls[p] * inv;
      const f32x4 x0 = __builtin_nontemporal_load(src), x1 = __builtin_nontemporal_load(src + 1);
      a0 += w * x0;
      a1 += w * x1;
    }
  }
  u32x4 out = {pack_bf16(a0[0], a0[1]), pack_bf16(a0[2], a0[3]), pack_bf16(a1[0], a1[1]), pack_bf16(a1[2], a1[3])};
  *reinterpret_cast<u32x4*>(o + off / 2) = out;
  if (c8 == 0) lse[(int64_t)h * tq + row] = tot > 0.f ? m_safe + __logf(tot) : -INFINITY;
}

// Every row: a 256-thread block covers 256 / (D/8) consecutive rows of ONE head so that the LSE reads (head-major)
// are contiguous.
template <int D>
__global__ __launch_bounds__(256) void merge_kernel(const float* __restrict__ o_part,
                                                    const float* __restrict__ lse_part, int n_parts,
                                                    int tq, int hq, uint32_t* __restrict__ o,
                                                    float* __restrict__ lse) {
  constexpr int TPR = D / 8;              // threads per (row, head)
  constexpr int ROWS = 256 / TPR;         // rows per block
  const int row = blockIdx.x * ROWS + threadIdx.x / TPR;
  if (row >= tq) return;
  merge_row_head<D>(o_part, lse_part, n_parts, tq, hq, o, lse, row, blockIdx.y, threadIdx.x % TPR);
}

// Direct mode: only the rows that the forward kernel did not finish itself are merged (the finished ones have
// state 2), and in a packed batch those are few.  A launch with a thread for every (row, head, 8 channels) spends its time starting waves that
// leave at once (9 us for 16 K rows x 32 heads, 58 us for 128 K rows); here a fixed number of waves walks the units
// (row, group of 64 / (D/8) heads) - wave w takes units w, w + W, ... - and reads the states of 64 of its units at a
// time, one per lane, so that a unit with nothing to do costs nothing.
template <int D>
__global__ __launch_bounds__(256) void merge_direct_kernel(const float* __restrict__ o_part,
                                                           const float* __restrict__ lse_part, int n_parts,
                                                           int tq, int hq, uint32_t* __restrict__ o,
                                                           float* __restrict__ lse, const uint8_t* __restrict__ q_state) {
  constexpr int TPR = D / 8;              // threads per (row, head)
  constexpr int HPW = 64 / TPR;           // heads a wave merges at once
  const int lane = threadIdx.x & 63;
  const int upr = (hq + HPW - 1) / HPW;   // units per row
  const int64_t n_units = (int64_t)tq * upr;
  const int64_t wstride = (int64_t)gridDim.x * 4;
  const int64_t w = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  for (int64_t u0 = w; u0 < n_units; u0 += 64 * wstride) {
    const int64_t mine = u0 + lane * wstride;
    const int st = mine < n_units ? q_state[mine / upr] : 2;
    uint64_t todo = __builtin_amdgcn_ballot_w64(st != 2);
    while (todo) {
      const int l = __builtin_ctzll(todo);
      todo &= todo - 1;
      const int64_t u = u0 + l * wstride;
      const int row = (int)(u / upr);
      const int h = (int)(u % upr) * HPW + lane / TPR;
      if (h < hq) merge_row_head<D>(o_part, lse_part, n_parts, tq, hq, o, lse, row, h, lane % TPR);
    }
  }
}

template <int D>
__global__ __launch_bounds__(256) void delta_kernel(const uint32_t* __restrict__ o,
                                                    const uint32_t* __restrict__ d_o, int tq, int hq,
                                                    float* __restrict__ delta) {
  constexpr int TPR = D / 8;
  constexpr int ROWS = 256 / TPR;
  const int h = blockIdx.y;
  const int row = blockIdx.x * ROWS + threadIdx.x / TPR;
  const int c8 = threadIdx.x % TPR;
  float s = 0.f;
  if (row < tq) {
    const int64_t off = (((int64_t)row * hq + h) * D + c8 * 8) / 2;
    const u32x4 a = *reinterpret_cast<const u32x4*>(o + off);
    const u32x4 b = *reinterpret_cast<const u32x4*>(d_o + off);
#pragma unroll
    for (int i = 0; i < 4; ++i) s += bf16_lo(a[i]) * bf16_lo(b[i]) + bf16_hi(a[i]) * bf16_hi(b[i]);
  }
#pragma unroll
  for (int off = TPR / 2; off > 0; off >>= 1) s += __shfl_xor(s, off, 64);
  if (row < tq && c8 == 0) delta[(int64_t)h * tq + row] = s;
}

__global__ __launch_bounds__(256) void finalize_kernel(const float* __restrict__ acc,
                                                       uint32_t* __restrict__ out, int64_t n8,
                                                       int64_t n) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n8; i += stride) {
    const f32x4* src = reinterpret_cast<const f32x4*>(acc) + 2 * i;
    const f32x4 x0 = src[0], x1 = src[1];
    u32x4 r = {pack_bf16(x0[0], x0[1]), pack_bf16(x0[2], x0[3]), pack_bf16(x1[0], x1[1]), pack_bf16(x1[2], x1[3])};
    reinterpret_cast<u32x4*>(out)[i] = r;
  }
  // tail (n not a multiple of 8): single elements, one thread
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    uint16_t* o16 = reinterpret_cast<uint16_t*>(out);
    for (int64_t i = n8 * 8; i < n; ++i) o16[i] = (uint16_t)bf16_rne(acc[i]);
  }
}

// Direct mode of the backward: the rows whose results were accumulated in fp32 (state 1) are converted, rows that
// no unit touched (state 0) are zero, rows written directly by their unit (state 2) are left alone.  One wave per
// row of dQ [tq], then dK [tkv], then dV [tkv]; wave w takes rows w, w + W, w + 2 W, ... and reads the states of 64 of
// its rows at a time, one per lane, so that the rows it has nothing to do for cost no trip to memory each.
__global__ __launch_bounds__(256) void finalize_direct_kernel(
    const uint8_t* __restrict__ q_state, const uint8_t* __restrict__ kv_state, int32_t tq, int32_t tkv,
    int32_t q_row_elems, int32_t kv_row_elems, const float* __restrict__ dq_acc, const float* __restrict__ dk_acc,
    const float* __restrict__ dv_acc, uint32_t* __restrict__ dq_out, uint32_t* __restrict__ dk_out,
    uint32_t* __restrict__ dv_out) {
  const int lane = threadIdx.x & 63;
  const int64_t n_rows = (int64_t)tq + 2 * (int64_t)tkv;
  const int64_t wstride = (int64_t)gridDim.x * 4;
  const int64_t w = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  auto state_of = [&](int64_t r) -> int {
    if (r >= n_rows) return 2;
    if (r < tq) return q_state[r];
    const int64_t kr = r - tq;
    return kv_state[kr >= tkv ? kr - tkv : kr];
  };
  for (int64_t r0 = w; r0 < n_rows; r0 += 64 * wstride) {
    const int mine = state_of(r0 + lane * wstride);                   // lane l: the wave's l-th row from r0 on
    uint64_t todo = __builtin_amdgcn_ballot_w64(mine != 2);
    while (todo) {
      const int l = __builtin_ctzll(todo);
      todo &= todo - 1;
      const int state = __builtin_amdgcn_readlane(mine, l);
      const int64_t r = r0 + l * wstride;
      int elems;
      const float* src;
      uint32_t* dst;
      if (r < tq) {
        elems = q_row_elems;
        src = dq_acc + r * q_row_elems; dst = dq_out + r * (q_row_elems / 2);
      } else {
        const bool is_v = r >= (int64_t)tq + tkv;
        const int64_t kr = r - tq - (is_v ? tkv : 0);
        elems = kv_row_elems;
        src = (is_v ? dv_acc : dk_acc) + kr * kv_row_elems; dst = (is_v ? dv_out : dk_out) + kr * (kv_row_elems / 2);
      }
      for (int32_t e = lane; e < elems / 8; e += 64) {
        u32x4 o = {0u, 0u, 0u, 0u};
        if (state == 1) {
          const f32x4* s4 = reinterpret_cast<const f32x4*>(src) + 2 * e;
          const f32x4 x0 = s4[0], x1 = s4[1];
          o = u32x4{pack_bf16(x0[0], x0[1]), pack_bf16(x0[2], x0[3]), pack_bf16(x1[0], x1[1]), pack_bf16(x1[2], x1[3])};
        }
        reinterpret_cast<u32x4*>(dst)[e] = o;
      }
    }
  }
}

}  // namespace
}  // namespace fcp

using fcp::fail;

static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

static int lse_merge(const float* o_part, const float* lse_part, int32_t n_parts, int32_t tq,
                     int32_t hq, int32_t head_dim, void* o, float* lse, void* stream, const uint8_t* q_state) {
  fcp::clear_error();
  if (!o_part || !lse_part || !o || !lse) return fail(FCP_ERR_INVALID_ARG, "fcp_lse_merge: null pointer");
  if (tq < 0 || hq < 1 || n_parts < 1) return fail(FCP_ERR_INVALID_ARG, "fcp_lse_merge: bad sizes");
  if (n_parts > fcp::kMaxParts) return fail(FCP_ERR_UNSUPPORTED, "fcp_lse_merge: n_parts %d > %d", n_parts, fcp::kMaxParts);
  if (head_dim != 64 && head_dim != 128) return fail(FCP_ERR_UNSUPPORTED, "fcp_lse_merge: head_dim %d not 64/128", head_dim);
  if (hq > 65535) return fail(FCP_ERR_UNSUPPORTED, "fcp_lse_merge: hq > 65535");
  if (!aligned16(o_part) || !aligned16(o)) return fail(FCP_ERR_INVALID_ARG, "fcp_lse_merge: o_part/o must be 16-byte aligned");
  if (tq == 0) return FCP_OK;
  hipStream_t st = (hipStream_t)stream;
  if (q_state) {
    const int hpw = 64 / (head_dim / 8);
    int64_t blocks = ((int64_t)tq * ((hq + hpw - 1) / hpw) + 3) / 4;
    if (blocks > 2048) blocks = 2048;
    if (blocks < 1) blocks = 1;
    if (head_dim == 128)
      hipLaunchKernelGGL(fcp::merge_direct_kernel<128>, dim3((unsigned)blocks), dim3(256), 0, st, o_part, lse_part, n_parts, tq, hq, (uint32_t*)o, lse, q_state);
    else
      hipLaunchKernelGGL(fcp::merge_direct_kernel<64>, dim3((unsigned)blocks), dim3(256), 0, st, o_part, lse_part, n_parts, tq, hq, (uint32_t*)o, lse, q_state);
  } else if (head_dim == 128) {
    dim3 grid((tq + 15) / 16, hq);
    hipLaunchKernelGGL(fcp::merge_kernel<128>, grid, dim3(256), 0, st, o_part, lse_part, n_parts, tq, hq, (uint32_t*)o, lse);
  } else {
    dim3 grid((tq + 31) / 32, hq);
    hipLaunchKernelGGL(fcp::merge_kernel<64>, grid, dim3(256), 0, st, o_part, lse_part, n_parts, tq, hq, (uint32_t*)o, lse);
  }
  FCP_HIP_CHECK(hipGetLastError());
  return FCP_OK;
}

extern "C" int fcp_lse_merge(const float* o_part, const float* lse_part, int32_t n_parts, int32_t tq,
                             int32_t hq, int32_t head_dim, void* o, float* lse, void* stream) {
  return lse_merge(o_part, lse_part, n_parts, tq, hq, head_dim, o, lse, stream, nullptr);
}

extern "C" int fcp_lse_merge_direct(const float* o_part, const float* lse_part, int32_t n_parts, int32_t tq,
                                    int32_t tkv, int32_t hq, int32_t head_dim, void* o, float* lse, void* scratch,
                                    int64_t n_work, void* stream) {
  if (!scratch || tkv < 1 || n_work < 0) {
    fcp::clear_error();
    return fail(FCP_ERR_INVALID_ARG, "fcp_lse_merge_direct: scratch is NULL or bad sizes");
  }
  return lse_merge(o_part, lse_part, n_parts, tq, hq, head_dim, o, lse, stream,
                   fcp::fwd_q_state(scratch, n_work, tq, tkv, n_parts));
}

extern "C" int fcp_attn_bwd_delta(const void* o, const void* d_o, int32_t tq, int32_t hq, int32_t head_dim,
                                  float* delta, void* stream) {
  fcp::clear_error();
  if (!o || !d_o || !delta) return fail(FCP_ERR_INVALID_ARG, "fcp_attn_bwd_delta: null pointer");
  if (tq < 0 || hq < 1 || hq > 65535) return fail(FCP_ERR_INVALID_ARG, "fcp_attn_bwd_delta: bad sizes");
  if (head_dim != 64 && head_dim != 128) return fail(FCP_ERR_UNSUPPORTED, "fcp_attn_bwd_delta: head_dim %d not 64/128", head_dim);
  if (!aligned16(o) || !aligned16(d_o)) return fail(FCP_ERR_INVALID_ARG, "fcp_attn_bwd_delta: o/d_o must be 16-byte aligned");
  if (tq == 0) return FCP_OK;
  hipStream_t st = (hipStream_t)stream;
  if (head_dim == 128) {
    dim3 grid((tq + 15) / 16, hq);
    hipLaunchKernelGGL(fcp::delta_kernel<128>, grid, dim3(256), 0, st, (const uint32_t*)o, (const uint32_t*)d_o, tq, hq, delta);
  } else {
    dim3 grid((tq + 31) / 32, hq);
    hipLaunchKernelGGL(fcp::delta_kernel<64>, grid, dim3(256), 0, st, (const uint32_t*)o, (const uint32_t*)d_o, tq, hq, delta);
  }
  FCP_HIP_CHECK(hipGetLastError());
  return FCP_OK;
}

extern "C" int fcp_grad_finalize(const float* acc, void* out_bf16, int64_t n, void* stream) {
  fcp::clear_error();
  if (!acc || !out_bf16) return fail(FCP_ERR_INVALID_ARG, "fcp_grad_finalize: null pointer");
  if (n < 0) return fail(FCP_ERR_INVALID_ARG, "fcp_grad_finalize: n < 0");
  if (!aligned16(acc) || !aligned16(out_bf16)) return fail(FCP_ERR_INVALID_ARG, "fcp_grad_finalize: pointers must be 16-byte aligned");
  if (n == 0) return FCP_OK;
  const int64_t n8 = n / 8;
  int64_t blocks = (n8 + 255) / 256;
  if (blocks > 8192) blocks = 8192;
  if (blocks < 1) blocks = 1;
  hipLaunchKernelGGL(fcp::finalize_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream, acc,
                     (uint32_t*)out_bf16, n8, n);
  FCP_HIP_CHECK(hipGetLastError());
  return FCP_OK;
}

extern "C" int fcp_grad_finalize_direct(const float* dq_acc, const float* dk_acc, const float* dv_acc, void* dq_out,
                                        void* dk_out, void* dv_out, void* scratch, int64_t n_work, int32_t tq,
                                        int32_t tkv, int32_t hq, int32_t hkv, int32_t head_dim, void* stream) {
  fcp::clear_error();
  if (!dq_acc || !dk_acc || !dv_acc || !dq_out || !dk_out || !dv_out || !scratch)
    return fail(FCP_ERR_INVALID_ARG, "fcp_grad_finalize_direct: null pointer");
  if (tq < 0 || tkv < 1 || hq < 1 || hkv < 1 || n_work < 0) return fail(FCP_ERR_INVALID_ARG, "fcp_grad_finalize_direct: bad sizes");
  if (head_dim != 64 && head_dim != 128) return fail(FCP_ERR_UNSUPPORTED, "fcp_grad_finalize_direct: head_dim %d not 64/128", head_dim);
  if (!aligned16(dq_acc) || !aligned16(dk_acc) || !aligned16(dv_acc) || !aligned16(dq_out) || !aligned16(dk_out) || !aligned16(dv_out))
    return fail(FCP_ERR_INVALID_ARG, "fcp_grad_finalize_direct: pointers must be 16-byte aligned");
  int64_t blocks = ((int64_t)tq + 2 * (int64_t)tkv + 3) / 4;
  if (blocks > 2048) blocks = 2048;     // a wave takes several rows; their states come in one load of 64
  hipLaunchKernelGGL(fcp::finalize_direct_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream,
                     fcp::bwd_q_state(scratch, n_work, tq, tkv, hq), fcp::bwd_kv_state(scratch, n_work, tq, tkv, hq), tq, tkv,
                     hq * head_dim, hkv * head_dim, dq_acc, dk_acc, dv_acc, (uint32_t*)dq_out, (uint32_t*)dk_out,
                     (uint32_t*)dv_out);
  FCP_HIP_CHECK(hipGetLastError());
  return FCP_OK;
}
