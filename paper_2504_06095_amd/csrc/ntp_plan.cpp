// Host-only part of the NTP library: status strings, shard plans and the
// sub-shard (segment) list of a reshard.  Pure integer arithmetic.
#include <algorithm>
#include <vector>

#include "ntp_internal.h"

extern "C" int ntp_version(void) { return 200; }

extern "C" const char* ntp_status_string(int status) {
  switch (status) {
    case NTP_OK: return "ok";
    case NTP_ERR_INVALID_ARG: return "invalid argument";
    case NTP_ERR_ALIGNMENT: return "pointer or leading dimension not aligned as required";
    case NTP_ERR_LAUNCH: return "HIP kernel launch failed";
    case NTP_ERR_UNSUPPORTED: return "size not supported";
    case NTP_ERR_NOT_PREPARED: return "reshard plan not prepared on this device";
    case NTP_ERR_NO_DEVICE: return "the handle was created with no device visible";
    case NTP_ERR_SCRATCH_TOO_SMALL: return "the shape needs more partial-sum room than the static scratch array has";
    default: return "unknown status";
  }
}

// Sec. 3.1: even-as-possible contiguous split, remainder on the lowest ranks.
extern "C" int ntp_shard_plan(int64_t dim, int32_t tp, int32_t rank, int64_t* offset,
                              int64_t* width) {
  if (dim < 0 || tp < 1 || rank < 0 || rank >= tp || !offset || !width) return NTP_ERR_INVALID_ARG;
  const int64_t base = dim / tp, rem = dim % tp;
  *width = base + (rank < rem ? 1 : 0);
  *offset = rank * base + std::min<int64_t>(rank, rem);
  return NTP_OK;
}

// Sec. 3.1, Eq. 4-6: heads are the unit; KV heads follow the query heads that read them.
extern "C" int ntp_attn_shard_plan(int32_t n_q, int32_t n_kv, int32_t head_dim, int32_t tp,
                                   int32_t rank, ntp_attn_plan_t* out) {
  if (!out || n_q < 1 || n_kv < 1 || head_dim < 1 || n_q % n_kv != 0) return NTP_ERR_INVALID_ARG;
  int64_t off = 0, cnt = 0;
  const int st = ntp_shard_plan(n_q, tp, rank, &off, &cnt);
  if (st != NTP_OK) return st;
  const int32_t group = n_q / n_kv;
  out->q_off = (int32_t)off;
  out->q_cnt = (int32_t)cnt;
  out->head_dim = head_dim;
  if (cnt == 0) {
    out->kv_off = 0;
    out->kv_cnt = 0;
  } else {
    const int32_t first = (int32_t)(off / group);
    const int32_t last = (int32_t)((off + cnt - 1) / group);
    out->kv_off = first;
    out->kv_cnt = last - first + 1;
  }
  out->w_qkv = (out->q_cnt + 2 * out->kv_cnt) * head_dim;
  out->w_o = out->q_cnt * head_dim;
  return NTP_OK;
}

namespace ntp {

int check_spec(const ntp_tensor_spec_t* spec, int32_t src_tp, int32_t dst_tp, int64_t* n_units) {
  if (!spec || src_tp < 1 || dst_tp < 1 || spec->rows < 0 || spec->cols < 0 || spec->unit < 1)
    return NTP_ERR_INVALID_ARG;
  if (spec->partition_dim != 0 && spec->partition_dim != 1) return NTP_ERR_INVALID_ARG;
  if (spec->elem_size != 2 && spec->elem_size != 4) return NTP_ERR_INVALID_ARG;
  const int64_t extent = spec->partition_dim == 0 ? spec->rows : spec->cols;
  if (extent % spec->unit != 0) return NTP_ERR_INVALID_ARG;
  *n_units = extent / spec->unit;
  if (spec->kind == NTP_KIND_QKV_GQA) {
    if (spec->n_q < 1 || spec->n_kv < 1 || spec->n_q % spec->n_kv != 0) return NTP_ERR_INVALID_ARG;
    if (*n_units != (int64_t)spec->n_q + 2 * (int64_t)spec->n_kv) return NTP_ERR_INVALID_ARG;
  } else if (spec->kind != NTP_KIND_PLAIN) {
    return NTP_ERR_INVALID_ARG;
  }
  return NTP_OK;
}

// A rank's shard as runs of consecutive logical units, in shard order.
int rank_runs(const ntp_tensor_spec_t* spec, int64_t n_units, int32_t tp, int32_t rank,
              std::vector<Run>* runs) {
  runs->clear();
  if (spec->kind == NTP_KIND_PLAIN) {
    int64_t off, w;
    const int st = ntp_shard_plan(n_units, tp, rank, &off, &w);
    if (st != NTP_OK) return st;
    if (w > 0) runs->push_back({off, w, 0});
    return NTP_OK;
  }
  ntp_attn_plan_t p;
  const int st = ntp_attn_shard_plan(spec->n_q, spec->n_kv, 1, tp, rank, &p);
  if (st != NTP_OK) return st;
  if (p.q_cnt > 0) {
    runs->push_back({p.q_off, p.q_cnt, 0});
    runs->push_back({(int64_t)spec->n_q + p.kv_off, p.kv_cnt, p.q_cnt});
    runs->push_back({(int64_t)spec->n_q + spec->n_kv + p.kv_off, p.kv_cnt, (int64_t)p.q_cnt + p.kv_cnt});
  }
  return NTP_OK;
}

int shard_units(const ntp_tensor_spec_t* spec, int64_t n_units, int32_t tp, int32_t rank,
                int64_t* units) {
  std::vector<Run> runs;
  const int st = rank_runs(spec, n_units, tp, rank, &runs);
  if (st != NTP_OK) return st;
  int64_t total = 0;
  for (const Run& r : runs) total += r.count;
  *units = total;
  return NTP_OK;
}

int build_segments(const ntp_tensor_spec_t* spec, int32_t src_tp, int32_t dst_tp,
                   std::vector<ntp_segment_t>* segs) {
  int64_t n_units = 0;
  int st = check_spec(spec, src_tp, dst_tp, &n_units);
  if (st != NTP_OK) return st;
  std::vector<std::vector<Run>> src(src_tp);
  for (int32_t r = 0; r < src_tp; ++r)
    if ((st = rank_runs(spec, n_units, src_tp, r, &src[r])) != NTP_OK) return st;
  segs->clear();
  std::vector<Run> dst;
  for (int32_t s = 0; s < dst_tp; ++s) {
    if ((st = rank_runs(spec, n_units, dst_tp, s, &dst)) != NTP_OK) return st;
    for (const Run& d : dst) {
      // cover [cur, end) from source ranks in ascending order: the first rank that
      // holds `cur` is the lowest one, which is the copy a replicated unit is read from
      int64_t cur = d.first;
      const int64_t end = d.first + d.count;
      for (int32_t r = 0; r < src_tp && cur < end; ++r) {
        for (const Run& a : src[r]) {
          if (cur < end && a.first <= cur && cur < a.first + a.count) {
            const int64_t stop = std::min(end, a.first + a.count);
            segs->push_back({r, s, a.local + (cur - a.first), d.local + (cur - d.first), stop - cur});
            cur = stop;
          }
        }
      }
      if (cur != end) return NTP_ERR_INVALID_ARG;  // cannot happen: every unit has a source rank
    }
  }
  return NTP_OK;
}

int build_segments_mapped(int64_t n_units, int32_t src_tp, const int32_t* src_map, int32_t dst_tp,
                          const int32_t* dst_map, std::vector<ntp_segment_t>* segs,
                          std::vector<int64_t>* src_units, std::vector<int64_t>* dst_units) {
  if (n_units < 0 || src_tp < 1 || dst_tp < 1 || (n_units > 0 && (!src_map || !dst_map))) return NTP_ERR_INVALID_ARG;
  src_units->assign(src_tp, 0);
  dst_units->assign(dst_tp, 0);
  // local position of every unit in its source shard, and the units of every destination shard
  std::vector<int64_t> src_local(n_units);
  std::vector<std::vector<int64_t>> dst_ids(dst_tp);
  for (int64_t u = 0; u < n_units; ++u) {
    const int32_t r = src_map[u], s = dst_map[u];
    if (r < 0 || r >= src_tp || s < 0 || s >= dst_tp) return NTP_ERR_INVALID_ARG;
    src_local[u] = (*src_units)[r]++;
    dst_ids[s].push_back(u);
    ++(*dst_units)[s];
  }
  segs->clear();
  for (int32_t s = 0; s < dst_tp; ++s) {
    const std::vector<int64_t>& ids = dst_ids[s];
    for (size_t j = 0; j < ids.size(); ++j) {
      const int64_t u = ids[j];
      const int32_t r = src_map[u];
      // extend the previous sub-shard when this unit follows it on both sides
      if (!segs->empty()) {
        ntp_segment_t& g = segs->back();
        if (g.dst_rank == s && g.src_rank == r && g.dst_unit + g.units == int64_t(j) &&
            g.src_unit + g.units == src_local[u]) {
          ++g.units;
          continue;
        }
      }
      segs->push_back({r, s, src_local[u], int64_t(j), 1});
    }
  }
  return NTP_OK;
}

}  // namespace ntp

// Sec. 3.1 "Shard-mapping algorithm", Alg. 1.
extern "C" int ntp_comp_sync_plan(int64_t k, int32_t full_tp, int32_t reduced_tp, int32_t* comp_rank,
                                  int32_t* sync_rank) {
  if (k < 0 || reduced_tp < 1 || full_tp < reduced_tp || (k > 0 && (!comp_rank || !sync_rank)))
    return NTP_ERR_INVALID_ARG;
  const int64_t keep = k / full_tp;
  const int32_t n_off = full_tp - reduced_tp;
  int32_t turn = 0;
  for (int32_t i = 0; i < reduced_tp; ++i) {
    int64_t off = 0, w = 0;
    ntp_shard_plan(k, reduced_tp, i, &off, &w);
    for (int64_t j = 0; j < w; ++j) {
      sync_rank[off + j] = i;
      if (j < keep || n_off == 0) {
        comp_rank[off + j] = i;
      } else {
        comp_rank[off + j] = reduced_tp + turn;
        turn = turn + 1 == n_off ? 0 : turn + 1;
      }
    }
  }
  return NTP_OK;
}

extern "C" int ntp_reshard_segments(const ntp_tensor_spec_t* spec, int32_t src_tp, int32_t dst_tp,
                                    ntp_segment_t* out, int64_t max_segments, int64_t* count) {
  if (!count || max_segments < 0 || (max_segments > 0 && !out)) return NTP_ERR_INVALID_ARG;
  std::vector<ntp_segment_t> segs;
  const int st = ntp::build_segments(spec, src_tp, dst_tp, &segs);
  if (st != NTP_OK) return st;
  *count = (int64_t)segs.size();
  for (int64_t i = 0; i < std::min<int64_t>(max_segments, (int64_t)segs.size()); ++i) out[i] = segs[i];
  return NTP_OK;
}

// Where the rows of one source rank's gradient go: its sub-shards joined with the destination shards.
extern "C" int ntp_reshard_row_segments(const ntp_tensor_spec_t* spec, int32_t src_tp, int32_t src_rank,
                                        int32_t dst_tp, void* const* dst_shards, const int64_t* dst_ld,
                                        ntp_row_segment_t* out, int64_t max_segments, int64_t* count) {
  if (!count || max_segments < 0 || (max_segments > 0 && !out) || !dst_shards || !dst_ld) return NTP_ERR_INVALID_ARG;
  std::vector<ntp_segment_t> segs;
  const int st = ntp::build_segments(spec, src_tp, dst_tp, &segs);
  if (st != NTP_OK) return st;
  if (src_rank < 0 || src_rank >= src_tp || spec->partition_dim != 0 || spec->elem_size != 4) return NTP_ERR_INVALID_ARG;
  if (spec->kind == NTP_KIND_QKV_GQA) {
    // A KV head that several source ranks hold: each holder's gradient GEMM yields only its own query heads'
    // share, so storing one holder's rows would drop the others'.  That layout needs the separate pass
    // (ntp_replica_sum, then ntp_reshard_grad).
    ntp_attn_plan_t mine, other;
    if (ntp_attn_shard_plan(spec->n_q, spec->n_kv, 1, src_tp, src_rank, &mine) != NTP_OK) return NTP_ERR_INVALID_ARG;
    for (int32_t r = 0; r < src_tp && mine.kv_cnt > 0; ++r) {
      if (r == src_rank || ntp_attn_shard_plan(spec->n_q, spec->n_kv, 1, src_tp, r, &other) != NTP_OK || other.kv_cnt == 0) continue;
      if (other.kv_off < mine.kv_off + mine.kv_cnt && mine.kv_off < other.kv_off + other.kv_cnt) return NTP_ERR_UNSUPPORTED;
    }
  }
  int64_t n = 0;
  for (const ntp_segment_t& g : segs) {
    if (g.src_rank != src_rank || g.units == 0) continue;
    if (!dst_shards[g.dst_rank]) continue;  // not on this GPU
    if (dst_ld[g.dst_rank] < spec->cols) return NTP_ERR_INVALID_ARG;
    if (n < max_segments)
      out[n] = ntp_row_segment_t{g.src_unit * spec->unit, g.units * spec->unit,
                                 static_cast<float*>(dst_shards[g.dst_rank]) + g.dst_unit * spec->unit * dst_ld[g.dst_rank],
                                 dst_ld[g.dst_rank]};
    ++n;
  }
  *count = n;
  return NTP_OK;
}
