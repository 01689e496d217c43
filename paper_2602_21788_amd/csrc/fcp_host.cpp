// Host-side parts of libfcp: error reporting and the shard plan.
#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <tuple>
#include <vector>

#include "fcp_internal.h"

namespace fcp {

static thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

void clear_error() { g_err[0] = 0; }

}  // namespace fcp

extern "C" const char* fcp_last_error(void) { return fcp::g_err; }

// Zigzag shard plan.  The paper fixes only "split evenly over the d ranks" (Sec. 4.3) and
// "d is any positive integer" (Sec. 4.2); the 2d-chunk zigzag with the remainder spread over
// the first chunks is the load-balanced form of that split for a causal mask.
extern "C" int fcp_shard_plan(const int32_t* seq_lens, const int32_t* cp_degree,
                              const int32_t* base_rank, int32_t n_seqs, fcp_chunk_desc* chunks,
                              int64_t chunk_cap, int64_t* n_chunks, fcp_work_desc* work,
                              int64_t work_cap, int64_t* n_work) {
  using fcp::fail;
  fcp::clear_error();
  if (!seq_lens || !cp_degree || !n_chunks || !n_work || n_seqs < 0)
    return fail(FCP_ERR_INVALID_ARG, "fcp_shard_plan: null argument or negative n_seqs");
  int64_t total = 0;
  for (int32_t s = 0; s < n_seqs; ++s) {
    if (seq_lens[s] < 1) return fail(FCP_ERR_INVALID_ARG, "fcp_shard_plan: seq_lens[%d] = %d < 1", s, seq_lens[s]);
    if (cp_degree[s] < 1 || cp_degree[s] > (1 << 20))
      return fail(FCP_ERR_INVALID_ARG, "fcp_shard_plan: cp_degree[%d] = %d out of range", s, cp_degree[s]);
    if (base_rank && base_rank[s] < 0) return fail(FCP_ERR_INVALID_ARG, "fcp_shard_plan: base_rank[%d] < 0", s);
    total += seq_lens[s];
  }
  if (total > INT32_MAX) return fail(FCP_ERR_UNSUPPORTED, "fcp_shard_plan: more than 2^31-1 tokens");

  // Pass 1: chunk table in (seq, chunk) order.
  std::vector<fcp_chunk_desc> cs;
  std::vector<int64_t> first_chunk(n_seqs + 1, 0);   // index of a sequence's chunk 0 in `cs`
  for (int32_t s = 0; s < n_seqs; ++s) {
    const int32_t L = seq_lens[s], d = cp_degree[s], base = base_rank ? base_rank[s] : 0;
    first_chunk[s] = (int64_t)cs.size();
    if (d == 1) {
      cs.push_back({s, base, 0, 0, L, 0});
    } else {
      const int32_t n = 2 * d, quot = L / n, rem = L % n;
      int32_t start = 0;
      for (int32_t c = 0; c < n; ++c) {
        const int32_t len = quot + (c < rem ? 1 : 0);
        const int32_t local = c < d ? c : n - 1 - c;
        cs.push_back({s, base + local, c, start, len, 0});
        start += len;
      }
    }
  }
  first_chunk[n_seqs] = (int64_t)cs.size();

  // Rank-local packed offsets: per rank, sequences in input order, early chunk before late.
  std::vector<int64_t> order(cs.size());
  for (size_t i = 0; i < order.size(); ++i) order[i] = (int64_t)i;
  std::stable_sort(order.begin(), order.end(), [&](int64_t a, int64_t b) {
    return std::tie(cs[a].rank, cs[a].seq, cs[a].chunk) < std::tie(cs[b].rank, cs[b].seq, cs[b].chunk);
  });
  {
    int32_t cur_rank = -1, off = 0;
    for (int64_t idx : order) {
      if (cs[idx].rank != cur_rank) { cur_rank = cs[idx].rank; off = 0; }
      cs[idx].local_off = off;
      off += cs[idx].len;
    }
  }

  // Pass 2: work items.
  std::vector<fcp_work_desc> ws;
  for (int32_t s = 0; s < n_seqs; ++s) {
    const int32_t d = cp_degree[s];
    const fcp_chunk_desc* c0 = cs.data() + first_chunk[s];
    for (int32_t i = 0; i < d; ++i) {
      for (int32_t step = 0; step < d; ++step) {
        const int32_t j = ((i - step) % d + d) % d;            // owner of this step's KV
        const int32_t q_chunks[2] = {i, 2 * d - 1 - i};
        const int32_t kv_chunks[2] = {j, 2 * d - 1 - j};       // increasing, j < 2d-1-j
        const int32_t n_own = d == 1 ? 1 : 2;
        for (int32_t qa = 0; qa < n_own; ++qa) {
          const fcp_chunk_desc& qc = c0[d == 1 ? 0 : q_chunks[qa]];
          if (qc.len == 0) continue;
          fcp_work_desc w{};
          w.seq = s; w.rank = qc.rank; w.step = step;
          w.q_local_off = qc.local_off; w.q_seq_start = qc.seq_start; w.q_len = qc.len;
          for (int32_t kb = 0; kb < n_own; ++kb) {
            const int32_t b = d == 1 ? 0 : kv_chunks[kb];
            if (b > qc.chunk || c0[b].len == 0) continue;      // later chunk: fully masked
            w.k_seq_start[w.n_seg] = c0[b].seq_start;
            w.k_len[w.n_seg] = c0[b].len;
            ++w.n_seg;
          }
          if (w.n_seg > 0) ws.push_back(w);
        }
      }
    }
  }
  std::stable_sort(ws.begin(), ws.end(), [](const fcp_work_desc& a, const fcp_work_desc& b) {
    return std::tie(a.rank, a.step, a.seq, a.q_seq_start) < std::tie(b.rank, b.step, b.seq, b.q_seq_start);
  });

  *n_chunks = (int64_t)cs.size();
  *n_work = (int64_t)ws.size();
  if ((chunks && chunk_cap < *n_chunks) || (work && work_cap < *n_work))
    return fail(FCP_ERR_CAPACITY, "fcp_shard_plan: need %lld chunk and %lld work entries",
                (long long)*n_chunks, (long long)*n_work);
  if (chunks)
    for (size_t i = 0; i < order.size(); ++i) chunks[i] = cs[order[i]];
  if (work) std::copy(ws.begin(), ws.end(), work);
  return FCP_OK;
}
