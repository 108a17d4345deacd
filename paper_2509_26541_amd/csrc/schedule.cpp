// tasp_schedule(N, rank): K_N ring decomposition (Sec. 3.1.2, Algorithm 1) or the multi-node
// (m-K_m-m)^u scheme (Sec. 3.1.3), routing tables (Algorithm 2), arrival order of the Multi-Ring
// AllGather (Sec. 3.2.2, Fig. 4) and sub-chunk placement (Sec. 3.2.3, eq. (3)-(6)).  Host code,
// integers only.
#include "schedule.hpp"

#include <algorithm>
#include <new>

namespace {

// Vertex sequence 0, 1, m-1, 2, m-2, ... on Z_m.  Its m cyclic translates are Hamiltonian paths in
// which every ordered pair of vertices is adjacent exactly once (a row-complete Latin square).
int32_t zigzag_at(int32_t t, int32_t m) {
  if (t == 0) return 0;
  return (t & 1) ? (t + 1) / 2 : m - t / 2;
}

// Algorithm 1.  Cycle i (i < n-2) on the n-1 vertices {0..n-2} is the new vertex n-2 followed by
// translate i of the zig-zag path on Z_{n-2}.  One arc is cut out of every cycle (chosen by the
// shift table) such that the cut arcs chain into one more Hamiltonian path; all n-1 paths are then
// closed through vertex n-1.
void decompose(int32_t n, std::vector<int32_t>& rings) {
  const int32_t m = n - 2;        // vertices of the zig-zag square
  const int32_t len = n - 1;      // length of an initial cycle
  const int32_t k = n / 4 - 1;
  rings.assign(static_cast<size_t>(n - 1) * n, -1);
  std::vector<int32_t> next_cut(len, -1);   // tail -> head of every cut arc
  for (int32_t i = 0; i < m; ++i) {
    int32_t shift = 2 * k;
    if (i == 0) shift = 1;
    else if (i == k + 1) shift = 4 * k + 2;
    else if (i == 2 * k + 2) shift = 3;
    else if (i == 3 * k + 2) shift = 4 * k;
    int32_t* ring = &rings[static_cast<size_t>(i) * n];
    for (int32_t j = 0; j < len; ++j) {
      const int32_t idx = (j + shift) % len;             // position in the unrotated cycle
      ring[j] = (idx == 0) ? n - 2 : (i + zigzag_at(idx - 1, m)) % m;
    }
    ring[len] = n - 1;
    next_cut[ring[len - 1]] = ring[0];
  }
  int32_t* last = &rings[static_cast<size_t>(m) * n];
  int32_t v = n - 2;
  for (int32_t j = 0; j < len; ++j) {
    last[j] = v;
    v = (v >= 0 && v < len) ? next_cut[v] : -1;
  }
  last[len] = n - 1;
}

// Sec. 3.1.3: every node (ranks c*m .. c*m+m-1) is cut into the m zig-zag paths; ring i runs through
// path i of node 0, path i of node 1, ... and closes from the last node to the first.  The paths of
// a node use each of its m(m-1) arcs once, and because every rank starts one path and ends one
// path, it sends to the next node once and receives from the previous node once.
void chain_nodes(int32_t m, int32_t u, std::vector<int32_t>& rings) {
  const int32_t n = m * u;
  rings.assign(static_cast<size_t>(m) * n, -1);
  for (int32_t i = 0; i < m; ++i)
    for (int32_t c = 0; c < u; ++c)
      for (int32_t t = 0; t < m; ++t)
        rings[static_cast<size_t>(i) * n + c * m + t] = c * m + (i + zigzag_at(t, m)) % m;
}

void fill_k4(std::vector<int32_t>& rings) {
  // K_4 has six directed Hamiltonian cycles and no three of them are arc-disjoint; this triple
  // repeats two arcs (0->1, 2->3) and leaves two unused (0->3, 2->1), the least possible.
  static const int32_t r[12] = {0, 1, 2, 3, 0, 1, 3, 2, 0, 2, 3, 1};
  rings.assign(r, r + 12);
}

}  // namespace

namespace tasp {

int n_query_blocks(int32_t mask_mode) { return mask_mode == TASP_MASK_ZIGZAG_CAUSAL ? 2 : 1; }

int check_sequence(const tasp_schedule& s, int64_t S, int32_t mask_mode) {
  if (mask_mode != TASP_MASK_FULL && mask_mode != TASP_MASK_ZIGZAG_CAUSAL) return TASP_EINVAL;
  const int64_t div = (mask_mode == TASP_MASK_FULL) ? s.n : 2 * static_cast<int64_t>(s.n);
  if (S <= 0 || S % div != 0) return TASP_EINVAL;
  return TASP_OK;
}

int query_block(const tasp_schedule& s, int64_t S, int32_t mask_mode, int32_t q_block, QueryBlock* out) {
  int st = check_sequence(s, S, mask_mode);
  if (st != TASP_OK) return st;
  if (q_block < 0 || q_block >= n_query_blocks(mask_mode)) return TASP_EINVAL;
  if (mask_mode == TASP_MASK_FULL) {
    const int64_t L = S / s.n;
    *out = {0, L, s.rank * L};
  } else {
    const int64_t H = S / (2 * static_cast<int64_t>(s.n));
    if (q_block == 0) *out = {0, H, s.rank * H};
    else *out = {H, H, S - (s.rank + 1) * H};
  }
  return TASP_OK;
}

static void piece_bounds(int64_t len, int32_t m, int32_t i, int64_t* a, int64_t* b) {
  *a = (static_cast<int64_t>(i) * len) / m;
  *b = (static_cast<int64_t>(i + 1) * len) / m;
}

static int subchunk(const tasp_schedule& s, int64_t S, int32_t mask_mode, int32_t ring, int32_t src,
                    int64_t r[4]) {
  const int32_t m = s.n_rings;
  int64_t a, b;
  if (mask_mode == TASP_MASK_FULL) {
    const int64_t L = S / s.n;
    piece_bounds(L, m, ring, &a, &b);
    r[0] = src * L + a;
    r[1] = src * L + b;
    return 1;
  }
  const int64_t H = S / (2 * static_cast<int64_t>(s.n));
  piece_bounds(H, m, ring, &a, &b);
  r[0] = src * H + a;            // eq. (5)
  r[1] = src * H + b;
  r[2] = S - src * H - b;        // eq. (6): the same piece counted from the end of the sequence
  r[3] = S - src * H - a;
  return 2;
}

// The key ranges a rank holds at `step`, in concatenation order.  With a query block they are
// filtered and marked by what the block can see; without one (q_block < 0) every range is listed.
static int arriving_ranges(const tasp_schedule& s, int64_t S, int32_t mask_mode, int32_t order, int32_t step,
                           int32_t q_block, std::vector<Segment>* out) {
  QueryBlock qb{0, 0, 0};
  int st = q_block >= 0 ? query_block(s, S, mask_mode, q_block, &qb) : check_sequence(s, S, mask_mode);
  if (st != TASP_OK) return st;
  if (step < 0 || step >= s.n) return TASP_EINVAL;
  if (order != TASP_ORDER_TASP && order != TASP_ORDER_RING) return TASP_EINVAL;
  const bool causal = mask_mode == TASP_MASK_ZIGZAG_CAUSAL;
  const bool filter = causal && q_block >= 0;
  const int64_t q_first = qb.pos0, q_last = qb.pos0 + qb.rows - 1;
  out->clear();
  auto push = [&](int64_t a, int64_t b) {
    if (a >= b) return;
    int32_t diag = 0;
    if (filter) {
      if (a > q_last) return;                 // hidden from every row of the block
      diag = (b - 1 > q_first) ? 1 : 0;       // some row sees only part of it
    }
    if (!out->empty() && out->back().end == a && out->back().diag == diag) out->back().end = b;
    else out->push_back({a, b, diag});
  };
  if (order == TASP_ORDER_TASP) {
    const int32_t m = s.n_rings;
    for (int32_t ring = 0; ring < m; ++ring) {
      const int32_t src = s.arrival[static_cast<size_t>(step) * m + ring];
      int64_t r[4];
      const int cnt = subchunk(s, S, mask_mode, ring, src, r);
      for (int c = 0; c < cnt; ++c) push(r[2 * c], r[2 * c + 1]);
    }
  } else {
    // Ring / Zig-zag Ring Attention: the whole chunk of rank (r - step) mod N arrives at once.
    const int32_t src = ((s.rank - step) % s.n + s.n) % s.n;
    if (!causal) {
      const int64_t L = S / s.n;
      push(src * L, (src + 1) * L);
    } else {
      const int64_t H = S / (2 * static_cast<int64_t>(s.n));
      push(src * H, (src + 1) * H);
      push(S - (src + 1) * H, S - src * H);
    }
  }
  return TASP_OK;
}

int step_segments(const tasp_schedule& s, int64_t S, int32_t mask_mode, int32_t order, int32_t step,
                  int32_t q_block, std::vector<Segment>* out) {
  if (q_block < 0) return TASP_EINVAL;
  return arriving_ranges(s, S, mask_mode, order, step, q_block, out);
}

int step_key_ranges(const tasp_schedule& s, int64_t S, int32_t mask_mode, int32_t order, int32_t step,
                    std::vector<Segment>* out) {
  return arriving_ranges(s, S, mask_mode, order, step, -1, out);
}

}  // namespace tasp

// ------------------------------------------------------------------------------------------------
// C ABI
// ------------------------------------------------------------------------------------------------
extern "C" {

const char* tasp_strerror(int status) {
  switch (status) {
    case TASP_OK: return "ok";
    case TASP_EINVAL: return "invalid argument";
    case TASP_EUNSUPPORTED_N: return "no ring decomposition for this number of ranks (need 4, or >= 8 and divisible by 4)";
    case TASP_EUNSUPPORTED_SHAPE: return "unsupported head dimension, dtype or size";
    case TASP_EALIGN: return "device pointer not 16-byte aligned";
    case TASP_EWORKSPACE: return "workspace missing or too small";
    case TASP_EHIP: return "HIP call or kernel launch failed";
    case TASP_ENOMEM: return "host allocation failed";
    default: return "unknown status";
  }
}

// Algorithm 2 and the arrival order, from the ring table of s.
static void derive_tables(tasp_schedule* s) {
  const int32_t n = s->n, m = s->n_rings, rank = s->rank;
  // Algorithm 2: highest ring first so that the lower id survives on a shared arc (N == 4).
  s->out_mapping.assign(static_cast<size_t>(n) * n, -1);
  s->in_mapping.assign(static_cast<size_t>(n) * n, -1);
  std::vector<int32_t> load(static_cast<size_t>(n) * n, 0);
  for (int32_t i = m - 1; i >= 0; --i) {
    const int32_t* ring = &s->rings[static_cast<size_t>(i) * n];
    for (int32_t j = 0; j < n; ++j) {
      const int32_t u = ring[j], v = ring[(j + 1) % n];
      s->out_mapping[static_cast<size_t>(u) * n + v] = i;
      s->in_mapping[static_cast<size_t>(v) * n + u] = i;
      ++load[static_cast<size_t>(u) * n + v];
    }
  }
  s->max_arc_load = *std::max_element(load.begin(), load.end());

  // Arrival order: on ring i the sub-chunk seen at step s started s hops upstream.
  s->arrival.assign(static_cast<size_t>(n) * m, -1);
  for (int32_t i = 0; i < m; ++i) {
    const int32_t* ring = &s->rings[static_cast<size_t>(i) * n];
    int32_t pos = 0;
    while (pos < n && ring[pos] != rank) ++pos;
    for (int32_t step = 0; step < n; ++step)
      s->arrival[static_cast<size_t>(step) * m + i] = ring[((pos - step) % n + n) % n];
  }
}

int tasp_schedule_create(int32_t n_ranks, int32_t rank, tasp_schedule_t** out) {
  if (out == nullptr) return TASP_EINVAL;
  *out = nullptr;
  if (n_ranks < 2 || rank < 0 || rank >= n_ranks) return TASP_EINVAL;
  if (n_ranks != 4 && (n_ranks < 8 || n_ranks % 4 != 0)) return TASP_EUNSUPPORTED_N;
  if (n_ranks > 4096) return TASP_EUNSUPPORTED_N;
  tasp_schedule* s = new (std::nothrow) tasp_schedule;
  if (s == nullptr) return TASP_ENOMEM;
  try {
    s->n = n_ranks;
    s->n_rings = n_ranks - 1;
    s->rank = rank;
    if (n_ranks == 4) fill_k4(s->rings); else decompose(n_ranks, s->rings);
    derive_tables(s);
  } catch (...) {
    delete s;
    return TASP_ENOMEM;
  }
  *out = s;
  return TASP_OK;
}

int tasp_schedule_create_multinode(int32_t ranks_per_node, int32_t n_nodes, int32_t rank, tasp_schedule_t** out) {
  if (out == nullptr) return TASP_EINVAL;
  *out = nullptr;
  if (ranks_per_node < 1 || n_nodes < 1 || ranks_per_node > 4096 || n_nodes > 4096) return TASP_EINVAL;
  const int32_t n = ranks_per_node * n_nodes;
  if (rank < 0 || rank >= n) return TASP_EINVAL;
  // the zig-zag paths need an even node size; with one node the closing arcs would repeat arcs of the paths
  if (ranks_per_node % 2 != 0 || n_nodes < 2 || n > 4096) return TASP_EUNSUPPORTED_N;
  tasp_schedule* s = new (std::nothrow) tasp_schedule;
  if (s == nullptr) return TASP_ENOMEM;
  try {
    s->n = n;
    s->n_rings = ranks_per_node;
    s->rank = rank;
    chain_nodes(ranks_per_node, n_nodes, s->rings);
    derive_tables(s);
  } catch (...) {
    delete s;
    return TASP_ENOMEM;
  }
  *out = s;
  return TASP_OK;
}

void tasp_schedule_destroy(tasp_schedule_t* s) { delete s; }

int32_t tasp_schedule_n_ranks(const tasp_schedule_t* s) { return s ? s->n : 0; }
int32_t tasp_schedule_rank(const tasp_schedule_t* s) { return s ? s->rank : -1; }
int32_t tasp_schedule_n_rings(const tasp_schedule_t* s) { return s ? s->n_rings : 0; }
int32_t tasp_schedule_max_arc_load(const tasp_schedule_t* s) { return s ? s->max_arc_load : 0; }
const int32_t* tasp_schedule_rings(const tasp_schedule_t* s) { return s ? s->rings.data() : nullptr; }
const int32_t* tasp_schedule_out_mapping(const tasp_schedule_t* s) { return s ? s->out_mapping.data() : nullptr; }
const int32_t* tasp_schedule_in_mapping(const tasp_schedule_t* s) { return s ? s->in_mapping.data() : nullptr; }
const int32_t* tasp_schedule_arrival(const tasp_schedule_t* s) { return s ? s->arrival.data() : nullptr; }

int tasp_subchunk_ranges(const tasp_schedule_t* s, int64_t S, int32_t mask_mode, int32_t ring,
                         int32_t src_rank, int64_t ranges[4], int32_t* n_ranges) {
  if (s == nullptr || ranges == nullptr || n_ranges == nullptr) return TASP_EINVAL;
  int st = tasp::check_sequence(*s, S, mask_mode);
  if (st != TASP_OK) return st;
  if (ring < 0 || ring >= s->n_rings || src_rank < 0 || src_rank >= s->n) return TASP_EINVAL;
  *n_ranges = tasp::subchunk(*s, S, mask_mode, ring, src_rank, ranges);
  return TASP_OK;
}

int tasp_step_segments(const tasp_schedule_t* s, int64_t S, int32_t mask_mode, int32_t order,
                       int32_t step, int32_t q_block, int64_t* seg, int32_t* diag, int32_t cap,
                       int32_t* n_seg) {
  if (s == nullptr || seg == nullptr || diag == nullptr || n_seg == nullptr || cap < 0) return TASP_EINVAL;
  std::vector<tasp::Segment> v;
  int st;
  try {
    st = tasp::step_segments(*s, S, mask_mode, order, step, q_block, &v);
  } catch (...) {
    return TASP_ENOMEM;
  }
  if (st != TASP_OK) return st;
  *n_seg = static_cast<int32_t>(v.size());
  if (static_cast<int64_t>(v.size()) > cap) return TASP_EINVAL;
  for (size_t i = 0; i < v.size(); ++i) {
    seg[2 * i] = v[i].start;
    seg[2 * i + 1] = v[i].end;
    diag[i] = v[i].diag;
  }
  return TASP_OK;
}

}  // extern "C"
