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

namespace {

// Full-attention spans of every sequence as (start, end) pairs in increasing order, and the mask they imply in
// the form the kernels use: a row at position i sees the keys 0 .. limit(i); a key at position j is seen by the
// rows from(j) .. L-1.  Outside a span both are the position itself (causal), inside a span its last and its
// first position.
struct SpanIndex {
  std::vector<std::vector<std::pair<int32_t, int32_t>>> by_seq;
  const std::pair<int32_t, int32_t>* find(int32_t seq, int32_t pos) const {
    const auto& v = by_seq[seq];
    auto it = std::upper_bound(v.begin(), v.end(), pos,
                               [](int32_t x, const std::pair<int32_t, int32_t>& sp) { return x < sp.first; });
    if (it == v.begin()) return nullptr;
    --it;
    return pos < it->second ? &*it : nullptr;
  }
  int32_t limit(int32_t seq, int32_t pos) const { auto sp = find(seq, pos); return sp ? sp->second - 1 : pos; }
  int32_t from(int32_t seq, int32_t pos) const { auto sp = find(seq, pos); return sp ? sp->first : pos; }
};

int build_span_index(const char* who, const int32_t* seq_lens, int32_t n_seqs, const fcp_span* spans, int32_t n_spans,
                     SpanIndex* out) {
  using fcp::fail;
  if (n_spans < 0 || (n_spans > 0 && !spans)) return fail(FCP_ERR_INVALID_ARG, "%s: bad span list", who);
  out->by_seq.assign((size_t)n_seqs, {});
  for (int32_t i = 0; i < n_spans; ++i) {
    const fcp_span& sp = spans[i];
    if (sp.seq < 0 || sp.seq >= n_seqs) return fail(FCP_ERR_INVALID_ARG, "%s: spans[%d].seq = %d out of range", who, i, sp.seq);
    if (sp.start < 0 || sp.len < 1 || (int64_t)sp.start + sp.len > (int64_t)seq_lens[sp.seq])
      return fail(FCP_ERR_INVALID_ARG, "%s: spans[%d] = [%d, +%d) leaves sequence %d of %d tokens", who, i, sp.start,
                  sp.len, sp.seq, seq_lens[sp.seq]);
    if (i > 0 && (spans[i - 1].seq > sp.seq || (spans[i - 1].seq == sp.seq && spans[i - 1].start + spans[i - 1].len > sp.start)))
      return fail(FCP_ERR_INVALID_ARG, "%s: spans must be sorted by (seq, start) and must not overlap (entry %d)", who, i);
    out->by_seq[sp.seq].emplace_back(sp.start, sp.start + sp.len);
  }
  return FCP_OK;
}

}  // namespace

// Zigzag shard plan.  The paper fixes only an even split of every sequence over the d ranks of its group (Sec. 4.3)
// and that d may be any positive integer (Sec. 4.2); the 2d-chunk zigzag with the remainder spread over
// the first chunks is the load-balanced form of that split for a causal mask.  With full-attention
// spans (Sec. 4.3, time estimation) the chunks stay the same and a query chunk additionally gets the
// later key chunks that a span reaching over the chunk border makes visible.
static int shard_plan(const char* who, const int32_t* seq_lens, const int32_t* cp_degree,
                      const int32_t* base_rank, int32_t n_seqs, const fcp_span* spans, int32_t n_spans,
                      fcp_chunk_desc* chunks, int64_t chunk_cap, int64_t* n_chunks, fcp_work_desc* work,
                      int64_t work_cap, int64_t* n_work) {
  using fcp::fail;
  fcp::clear_error();
  if (!seq_lens || !cp_degree || !n_chunks || !n_work || n_seqs < 0)
    return fail(FCP_ERR_INVALID_ARG, "%s: null argument or negative n_seqs", who);
  int64_t total = 0;
  for (int32_t s = 0; s < n_seqs; ++s) {
    if (seq_lens[s] < 1) return fail(FCP_ERR_INVALID_ARG, "%s: seq_lens[%d] = %d < 1", who, s, seq_lens[s]);
    if (cp_degree[s] < 1 || cp_degree[s] > (1 << 20))
      return fail(FCP_ERR_INVALID_ARG, "%s: cp_degree[%d] = %d out of range", who, s, cp_degree[s]);
    if (base_rank && base_rank[s] < 0) return fail(FCP_ERR_INVALID_ARG, "%s: base_rank[%d] < 0", who, s);
    total += seq_lens[s];
  }
  if (total > INT32_MAX) return fail(FCP_ERR_UNSUPPORTED, "%s: more than 2^31-1 tokens", who);
  SpanIndex mask;
  if (int rc = build_span_index(who, seq_lens, n_seqs, spans, n_spans, &mask)) return rc;

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
          const int32_t last_seen = mask.limit(s, qc.seq_start + qc.len - 1);   // by the chunk's last row, hence by any
          for (int32_t kb = 0; kb < n_own; ++kb) {
            const int32_t b = d == 1 ? 0 : kv_chunks[kb];
            if (c0[b].len == 0 || c0[b].seq_start > last_seen) continue;   // empty, or fully masked (a later chunk)
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
    return fail(FCP_ERR_CAPACITY, "%s: need %lld chunk and %lld work entries", who,
                (long long)*n_chunks, (long long)*n_work);
  if (chunks)
    for (size_t i = 0; i < order.size(); ++i) chunks[i] = cs[order[i]];
  if (work) std::copy(ws.begin(), ws.end(), work);
  return FCP_OK;
}

extern "C" int fcp_shard_plan(const int32_t* seq_lens, const int32_t* cp_degree,
                              const int32_t* base_rank, int32_t n_seqs, fcp_chunk_desc* chunks,
                              int64_t chunk_cap, int64_t* n_chunks, fcp_work_desc* work,
                              int64_t work_cap, int64_t* n_work) {
  return shard_plan("fcp_shard_plan", seq_lens, cp_degree, base_rank, n_seqs, nullptr, 0, chunks, chunk_cap, n_chunks,
                    work, work_cap, n_work);
}

extern "C" int fcp_shard_plan_mixed(const int32_t* seq_lens, const int32_t* cp_degree,
                                    const int32_t* base_rank, int32_t n_seqs, const fcp_span* spans,
                                    int32_t n_spans, fcp_chunk_desc* chunks, int64_t chunk_cap,
                                    int64_t* n_chunks, fcp_work_desc* work, int64_t work_cap, int64_t* n_work) {
  return shard_plan("fcp_shard_plan_mixed", seq_lens, cp_degree, base_rank, n_seqs, spans, n_spans, chunks, chunk_cap,
                    n_chunks, work, work_cap, n_work);
}

extern "C" int fcp_mask_tables(const int32_t* seq_lens, int32_t n_seqs, const fcp_span* spans, int32_t n_spans,
                               const fcp_chunk_desc* chunks, int64_t n_chunks, int32_t rank, int32_t* q_limit,
                               int64_t q_limit_cap, int64_t* n_q, int32_t* k_from, float* eta) {
  using fcp::fail;
  fcp::clear_error();
  const char* who = "fcp_mask_tables";
  if (!seq_lens || n_seqs < 0 || n_chunks < 0 || (n_chunks > 0 && !chunks))
    return fail(FCP_ERR_INVALID_ARG, "%s: null argument or negative count", who);
  for (int32_t s = 0; s < n_seqs; ++s)
    if (seq_lens[s] < 1) return fail(FCP_ERR_INVALID_ARG, "%s: seq_lens[%d] = %d < 1", who, s, seq_lens[s]);
  SpanIndex mask;
  if (int rc = build_span_index(who, seq_lens, n_seqs, spans, n_spans, &mask)) return rc;
  int64_t rows = 0;
  for (int64_t i = 0; i < n_chunks; ++i) {
    const fcp_chunk_desc& c = chunks[i];
    if (c.rank != rank) continue;
    if (c.seq < 0 || c.seq >= n_seqs || c.seq_start < 0 || c.len < 0 || c.local_off < 0 ||
        (int64_t)c.seq_start + c.len > (int64_t)seq_lens[c.seq])
      return fail(FCP_ERR_INVALID_ARG, "%s: chunks[%lld] does not fit its sequence", who, (long long)i);
    rows = std::max<int64_t>(rows, (int64_t)c.local_off + c.len);
  }
  if (n_q) *n_q = rows;
  if (q_limit) {
    if (q_limit_cap < rows) return fail(FCP_ERR_CAPACITY, "%s: q_limit needs %lld entries", who, (long long)rows);
    for (int64_t i = 0; i < n_chunks; ++i) {
      const fcp_chunk_desc& c = chunks[i];
      if (c.rank != rank) continue;
      for (int32_t r = 0; r < c.len; ++r) q_limit[c.local_off + r] = mask.limit(c.seq, c.seq_start + r);
    }
  }
  int64_t t0 = 0;
  for (int32_t s = 0; s < n_seqs; ++s) {
    const int64_t L = seq_lens[s];
    if (k_from)
      for (int32_t pos = 0; pos < L; ++pos) k_from[t0 + pos] = mask.from(s, pos);
    if (eta) {
      int64_t extra = 0;       // pairs above the diagonal: n (n - 1) / 2 per span of n tokens
      for (const auto& sp : mask.by_seq[s]) extra += (int64_t)(sp.second - sp.first) * (sp.second - sp.first - 1) / 2;
      eta[s] = (float)((double)extra / (double)(L * (L + 1) / 2));
    }
    t0 += L;
  }
  return FCP_OK;
}
