// Host-side memory passes on an operator list (Sections 3.1.4 and 3.1.5 of the paper): the liveness-based
// memory estimate, operator scheduling by the p - c rule, and rematerialisation under a byte budget, plus
// the operator list of a stack of this library's transformer layers, from which the per-layer
// rematerialisation bits of raf_layer_desc are planned.  No device code here.
#include <algorithm>
#include <cstdint>
#include <vector>

#include "raf_mi355.h"
#include "common.hpp"

namespace raf {
namespace {

struct Graph {
  int n_ops = 0, n_t = 0;
  std::vector<std::vector<int>> in, out;   // distinct tensor ids per op
  std::vector<double> lat;
  std::vector<int64_t> bytes;
  std::vector<uint8_t> remat_ok, persistent;
  std::vector<int> prod;                   // producing op of a tensor, -1 = external
};

bool load_graph(const raf_op_graph* g, Graph& G) {
  if (!g || g->n_ops < 0 || g->n_tensors < 0) return false;
  if (g->n_ops && (!g->in_begin || !g->out_begin || !g->latency)) return false;
  if (g->n_tensors && (!g->bytes || !g->flags)) return false;
  G.n_ops = g->n_ops;
  G.n_t = g->n_tensors;
  G.in.assign(G.n_ops, {});
  G.out.assign(G.n_ops, {});
  G.lat.assign(g->latency, g->latency + G.n_ops);
  G.bytes.assign(g->bytes, g->bytes + G.n_t);
  G.remat_ok.resize(G.n_t);
  G.persistent.resize(G.n_t);
  for (int t = 0; t < G.n_t; ++t) {
    if (G.bytes[t] < 0) return false;
    G.remat_ok[t] = g->flags[t] & RAF_TENSOR_REMAT_OK;
    G.persistent[t] = (g->flags[t] & RAF_TENSOR_PERSISTENT) ? 1 : 0;
  }
  G.prod.assign(G.n_t, -1);
  auto fill = [&](const int32_t* begin, const int32_t* ids, int k, std::vector<int>& dst) {
    if (begin[k] < 0 || begin[k + 1] < begin[k]) return false;
    if (begin[k + 1] > begin[k] && !ids) return false;
    for (int q = begin[k]; q < begin[k + 1]; ++q) {
      if (ids[q] < 0 || ids[q] >= G.n_t) return false;
      if (std::find(dst.begin(), dst.end(), (int)ids[q]) == dst.end()) dst.push_back(ids[q]);
    }
    return true;
  };
  for (int k = 0; k < G.n_ops; ++k) {
    if (!(G.lat[k] >= 0.0)) return false;
    if (!fill(g->in_begin, g->in_ids, k, G.in[k]) || !fill(g->out_begin, g->out_ids, k, G.out[k])) return false;
    for (int t : G.out[k]) {
      if (G.prod[t] >= 0) return false;   // two producers
      G.prod[t] = k;
    }
  }
  return true;
}

// an item of an execution sequence: k >= 0 runs op k, -1 - t replays the producer of t for t alone
inline const std::vector<int>& item_in(const Graph& G, int item) { return G.in[item >= 0 ? item : G.prod[-1 - item]]; }

bool item_valid(const Graph& G, int item) {
  if (item >= 0) return item < G.n_ops;
  const int t = -1 - item;
  return t < G.n_t && G.prod[t] >= 0;
}

struct Span { int first, last; };

// Liveness of every tensor over a sequence: one span per materialisation, from the item that writes the tensor
// to the last item that reads it before it is written again (to the end for the last span of a persistent
// tensor).  False if an item reads a tensor that does not exist yet.
bool live_spans(const Graph& G, const std::vector<int>& seq, std::vector<std::vector<Span>>& spans) {
  const int n = (int)seq.size();
  spans.assign(G.n_t, {});
  for (int t = 0; t < G.n_t; ++t)
    if (G.prod[t] < 0 && n > 0) spans[t].push_back(Span{0, n - 1});
  for (int pos = 0; pos < n; ++pos) {
    const int item = seq[pos];
    for (int t : item_in(G, item)) {
      if (G.prod[t] < 0) continue;
      if (spans[t].empty()) return false;
      spans[t].back().last = pos;
    }
    if (item >= 0) {
      for (int t : G.out[item]) spans[t].push_back(Span{pos, pos});
    } else {
      spans[-1 - item].push_back(Span{pos, pos});
    }
  }
  for (int t = 0; t < G.n_t; ++t)
    if (G.prod[t] >= 0 && G.persistent[t] && !spans[t].empty()) spans[t].back().last = n - 1;
  return true;
}

void profile_of(const Graph& G, const std::vector<std::vector<Span>>& spans, int n, std::vector<int64_t>& mem) {
  std::vector<int64_t> delta(n + 1, 0);
  for (int t = 0; t < G.n_t; ++t)
    for (const Span& s : spans[t]) {
      delta[s.first] += G.bytes[t];
      delta[s.last + 1] -= G.bytes[t];
    }
  mem.assign(n, 0);
  int64_t run = 0;
  for (int pos = 0; pos < n; ++pos) {
    run += delta[pos];
    mem[pos] = run;
  }
}

bool alive_before(const std::vector<Span>& sp, int j) {   // materialised before item j and still alive when it runs
  for (const Span& s : sp)
    if (s.first < j && j <= s.last) return true;
  return false;
}

double total_latency(const Graph& G, const std::vector<int>& seq) {
  double total = 0.0;
  for (int item : seq) total += G.lat[item >= 0 ? item : G.prod[-1 - item]];
  return total;
}

struct PlanResult {
  std::vector<int> seq, ev_tensor, ev_pos;
  int64_t peak_before = 0, peak_after = 0;
  bool fits = true;
  double extra_latency = 0.0;
};

// Section 3.1.5.  The order is walked once; where the estimate exceeds the budget, the alive tensor with the
// lowest  latency(producer) * uses still to come / bytes  is dropped (ties: larger, then lower id) and a
// replay of its producer is put in front of its next reader, until the point fits or nothing qualifies.  A
// tensor qualifies if it may be regenerated, the current item does not touch it, its next reader is not the
// very next item, and every input of its producer is still alive where the replay goes (one operator is
// replayed, never a chain).
bool plan_remat(const Graph& G, int64_t budget, PlanResult& R) {
  R.seq.resize(G.n_ops);
  for (int k = 0; k < G.n_ops; ++k) R.seq[k] = k;
  std::vector<std::vector<Span>> spans;
  std::vector<int64_t> mem;
  if (!live_spans(G, R.seq, spans)) return false;
  profile_of(G, spans, (int)R.seq.size(), mem);
  R.peak_before = mem.empty() ? 0 : *std::max_element(mem.begin(), mem.end());
  const double base_latency = total_latency(G, R.seq);
  const size_t cap = 8 * (size_t)G.n_ops + 8;
  std::vector<char> busy(G.n_t, 0);
  for (size_t i = 0; i < R.seq.size(); ++i) {
    while (mem[i] > budget) {
      if (R.seq.size() >= cap) { R.fits = false; break; }
      const int item = R.seq[i];
      std::fill(busy.begin(), busy.end(), 0);
      for (int t : item_in(G, item)) busy[t] = 1;
      if (item >= 0) { for (int t : G.out[item]) busy[t] = 1; } else busy[-1 - item] = 1;
      int best = -1, best_at = -1;
      double best_cost = 0.0;
      for (int t = 0; t < G.n_t; ++t) {
        if (!G.remat_ok[t] || G.prod[t] < 0 || busy[t] || G.bytes[t] <= 0) continue;
        const Span* cover = nullptr;
        for (const Span& s : spans[t])
          if (s.first < (int)i && (int)i <= s.last) { cover = &s; break; }
        if (!cover) continue;
        int uses = 0, next = -1;
        for (int pos = (int)i + 1; pos <= cover->last; ++pos) {
          const std::vector<int>& in = item_in(G, R.seq[pos]);
          if (std::find(in.begin(), in.end(), t) != in.end()) {
            if (next < 0) next = pos;
            ++uses;
          }
        }
        if (uses == 0 || next == (int)i + 1) continue;
        bool inputs_alive = true;
        for (int s : G.in[G.prod[t]])
          if (G.prod[s] >= 0 && !alive_before(spans[s], next)) { inputs_alive = false; break; }
        if (!inputs_alive) continue;
        const double cost = G.lat[G.prod[t]] * (double)uses / (double)G.bytes[t];
        const bool better = best < 0 || cost < best_cost ||
                            (cost == best_cost && (G.bytes[t] > G.bytes[best] || (G.bytes[t] == G.bytes[best] && t < best)));
        if (better) { best = t; best_at = next; best_cost = cost; }
      }
      if (best < 0) { R.fits = false; break; }
      R.ev_tensor.push_back(best);
      R.ev_pos.push_back((int)i);
      R.seq.insert(R.seq.begin() + best_at, -1 - best);
      if (!live_spans(G, R.seq, spans)) return false;
      profile_of(G, spans, (int)R.seq.size(), mem);
    }
  }
  R.peak_after = mem.empty() ? 0 : *std::max_element(mem.begin(), mem.end());
  R.extra_latency = total_latency(G, R.seq) - base_latency;
  return true;
}

// ---- the operator list of a stack of layers, in the order raf_layer_fwd / raf_layer_bwd launch their kernels
struct StackGraph {
  std::vector<int32_t> in_begin{0}, in_ids, out_begin{0}, out_ids;
  std::vector<double> lat;
  std::vector<int64_t> bytes;
  std::vector<uint8_t> flags;
  std::vector<int32_t> owner_layer, owner_bit;   // per tensor: layer and raf_remat_bits value, or -1 / 0
  int add_tensor(int64_t b, uint8_t f, int layer = -1, int bit = 0) {
    bytes.push_back(b); flags.push_back(f); owner_layer.push_back(layer); owner_bit.push_back(bit);
    return (int)bytes.size() - 1;
  }
  void add_op(std::initializer_list<int> in, std::initializer_list<int> out, double latency) {
    for (int t : in) if (t >= 0) in_ids.push_back(t);
    for (int t : out) if (t >= 0) out_ids.push_back(t);
    in_begin.push_back((int32_t)in_ids.size());
    out_begin.push_back((int32_t)out_ids.size());
    lat.push_back(latency);
  }
};

// replay latencies in microseconds when the caller has no measured ones: the slower of 2MNK flops at 800 TFLOP/s
// (what these products reach on this chip) and the operand + result bytes at 4 TB/s
double product_estimate_us(double M, double N, double K, double e, double outs) {
  const double flops = 2.0 * M * N * K, bytes = e * (M * K + N * K + outs * M * N);
  return std::max(flops / 800e12, bytes / 4e12) * 1e6;
}

bool build_stack(const raf_layer_desc& d, int layers, const double* replay_us, StackGraph& S) {
  const bool bf16 = d.precision == RAF_BF16_AMP;
  const bool flash = attn_flash_supported(d), onchip = flash || attn_fused_supported(d);
  const double e = bf16 ? 2 : 4;
  const int64_t T = (int64_t)d.batch * d.seq, H = d.hidden, F = d.ffn;
  const int64_t TH = (int64_t)(T * H * e), TF = (int64_t)(T * F * e);
  const int64_t stat = T * 8, PS = onchip ? 0 : (int64_t)((double)d.batch * d.heads * d.seq * d.seq * e);
  // row statistics of the blockwise attention and the keep decisions of its dropout site: one tensor here
  const int64_t rowstat = flash ? (int64_t)d.batch * d.heads * d.seq * 4 + (int64_t)attn_flash_keep_bytes(d) : 0;
  double us[3];
  if (replay_us) {
    for (int i = 0; i < 3; ++i) {
      if (!(replay_us[i] >= 0.0)) return false;
      us[i] = replay_us[i];
    }
  } else {
    us[0] = product_estimate_us((double)T, 3.0 * H, (double)H, e, 1);
    // scores and context: 4 T S H flops, half of them under a causal mask
    us[1] = std::max(4.0 * T * d.seq * H * (d.causal ? 0.5 : 1.0) / 800e12, e * 4.0 * T * H / 4e12) * 1e6;
    us[2] = product_estimate_us((double)T, (double)F, (double)H, e, 2);
  }
  const uint8_t OK = RAF_TENSOR_REMAT_OK;
  struct LayerT { int x, n1, qkv, probs, ctx, lse, z1, ffn_in, st1, ffn1, z2, st2, y; };
  std::vector<LayerT> L(layers);
  int x = S.add_tensor(TH, 0);   // the stack's input: external
  for (int l = 0; l < layers; ++l) {
    LayerT& t = L[l];
    t.x = x;
    t.n1 = d.pre_ln ? S.add_tensor(TH, 0) : -1;
    t.st1 = S.add_tensor(stat, 0);
    if (d.pre_ln) S.add_op({t.x}, {t.n1, t.st1}, 0.0);
    t.qkv = S.add_tensor(3 * TH, OK, l, RAF_REMAT_QKV);
    S.add_op({d.pre_ln ? t.n1 : t.x}, {t.qkv}, us[0]);
    t.ctx = S.add_tensor(TH, onchip ? OK : 0, l, onchip ? RAF_REMAT_CTX : 0);
    t.lse = rowstat ? S.add_tensor(rowstat, 0) : -1;
    t.probs = PS ? S.add_tensor(2 * PS, 0) : -1;
    S.add_op({t.qkv}, {t.ctx, t.lse, t.probs}, us[1]);
    const int a1 = S.add_tensor(TH, 0);
    S.add_op({t.ctx}, {a1}, 0.0);
    t.z1 = S.add_tensor(TH, 0);
    t.ffn_in = S.add_tensor(TH, 0);
    t.st2 = S.add_tensor(stat, 0);
    if (d.pre_ln) S.add_op({a1, t.x}, {t.z1, t.ffn_in, t.st2}, 0.0);
    else S.add_op({a1, t.x}, {t.z1, t.ffn_in, t.st1}, 0.0);
    t.ffn1 = S.add_tensor(2 * TF, OK, l, RAF_REMAT_FFN1);
    S.add_op({t.ffn_in}, {t.ffn1}, us[2]);
    const int a2 = S.add_tensor(TH, 0);
    S.add_op({t.ffn1}, {a2}, 0.0);
    t.z2 = d.pre_ln ? -1 : S.add_tensor(TH, 0);
    t.y = S.add_tensor(TH, 0);
    if (d.pre_ln) S.add_op({a2, t.z1}, {t.y}, 0.0);
    else S.add_op({a2, t.ffn_in}, {t.y, t.z2, t.st2}, 0.0);
    x = t.y;
  }
  int dy = S.add_tensor(TH, 0);
  S.add_op({x}, {dy}, 0.0);   // loss seed
  for (int l = layers - 1; l >= 0; --l) {
    const LayerT& t = L[l];
    const int dz2 = d.pre_ln ? -1 : S.add_tensor(TH, 0), da2 = S.add_tensor(TH, 0);
    if (d.pre_ln) S.add_op({dy}, {da2}, 0.0);
    else S.add_op({dy, t.z2, t.st2}, {dz2, da2}, 0.0);
    const int du = S.add_tensor(TF, 0);
    S.add_op({da2, t.ffn1}, {du}, 0.0);
    const int dffn = S.add_tensor(TH, 0);
    S.add_op({du}, {dffn}, 0.0);
    const int dz1 = S.add_tensor(TH, 0), da1 = S.add_tensor(TH, 0);
    if (d.pre_ln) S.add_op({dffn, t.z1, t.st2, dy}, {dz1, da1}, 0.0);
    else S.add_op({dz2, dffn, t.z1, t.st1}, {dz1, da1}, 0.0);
    const int dc = S.add_tensor(TH, 0);
    S.add_op({da1}, {dc}, 0.0);
    const int dqkv = S.add_tensor(3 * TH, 0);
    if (flash) S.add_op({dc, t.qkv, t.ctx, t.lse}, {dqkv}, 0.0);
    else if (onchip) S.add_op({dc, t.qkv}, {dqkv}, 0.0);
    else S.add_op({dc, t.qkv, t.probs}, {dqkv}, 0.0);
    const int dx = S.add_tensor(TH, l == 0 ? RAF_TENSOR_PERSISTENT : 0);
    if (d.pre_ln) S.add_op({dqkv, dz1, t.x, t.st1}, {dx}, 0.0);
    else S.add_op({dqkv, dz1}, {dx}, 0.0);
    // the grouped weight-gradient launch closes the layer; gradients live in the caller's parameter-sized
    // buffers, outside the activation budget
    const int grads = S.add_tensor(0, RAF_TENSOR_PERSISTENT);
    S.add_op({da2, t.ffn1, du, t.ffn_in, dqkv, d.pre_ln ? t.n1 : t.x, da1, t.ctx}, {grads}, 0.0);
    dy = dx;
  }
  return true;
}

raf_op_graph view(const StackGraph& S) {
  raf_op_graph g{};
  g.n_ops = (int32_t)S.lat.size();
  g.n_tensors = (int32_t)S.bytes.size();
  g.in_begin = S.in_begin.data(); g.in_ids = S.in_ids.data();
  g.out_begin = S.out_begin.data(); g.out_ids = S.out_ids.data();
  g.latency = S.lat.data(); g.bytes = S.bytes.data(); g.flags = S.flags.data();
  return g;
}

}  // namespace
}  // namespace raf

using namespace raf;

extern "C" raf_status raf_memory_profile(const raf_op_graph* graph, const int32_t* sequence, int32_t seq_len,
                                         int64_t* mem_out) {
  Graph G;
  if (!load_graph(graph, G)) return RAF_EINVAL;
  std::vector<int> seq;
  if (sequence) {
    if (seq_len < 0) return RAF_EINVAL;
    seq.assign(sequence, sequence + seq_len);
  } else {
    seq.resize(G.n_ops);
    for (int k = 0; k < G.n_ops; ++k) seq[k] = k;
  }
  for (int item : seq)
    if (!item_valid(G, item)) return RAF_EINVAL;
  if (!seq.empty() && !mem_out) return RAF_EINVAL;
  std::vector<std::vector<Span>> spans;
  if (!live_spans(G, seq, spans)) return RAF_EINVAL;
  std::vector<int64_t> mem;
  profile_of(G, spans, (int)seq.size(), mem);
  std::copy(mem.begin(), mem.end(), mem_out);
  return RAF_OK;
}

extern "C" raf_status raf_schedule_ops(const raf_op_graph* graph, int32_t* order_out) {
  Graph G;
  if (!load_graph(graph, G)) return RAF_EINVAL;
  if (G.n_ops && !order_out) return RAF_EINVAL;
  // Section 3.1.4 as list scheduling: of the operators whose inputs exist, the one with the smallest p - c runs
  // next, p = bytes it produces, c = bytes released once it has run; ties in the given order
  std::vector<int> readers_left(G.n_t, 0);
  for (int k = 0; k < G.n_ops; ++k)
    for (int t : G.in[k]) ++readers_left[t];
  std::vector<char> done(G.n_ops, 0), exists(G.n_t, 0);
  for (int t = 0; t < G.n_t; ++t) exists[t] = G.prod[t] < 0;
  for (int step = 0; step < G.n_ops; ++step) {
    int best = -1;
    int64_t best_delta = 0;
    for (int k = 0; k < G.n_ops; ++k) {
      if (done[k]) continue;
      bool ready = true;
      for (int t : G.in[k]) ready = ready && exists[t];
      if (!ready) continue;
      int64_t delta = 0;
      for (int t : G.out[k]) {
        delta += G.bytes[t];
        if (readers_left[t] == 0 && !G.persistent[t]) delta -= G.bytes[t];   // nothing reads it: let go at once
      }
      for (int t : G.in[k])
        if (G.prod[t] >= 0 && !G.persistent[t] && readers_left[t] == 1) delta -= G.bytes[t];
      if (best < 0 || delta < best_delta) { best = k; best_delta = delta; }
    }
    if (best < 0) return RAF_EINVAL;   // a cycle, or an input that nothing produces before its reader
    done[best] = 1;
    order_out[step] = best;
    for (int t : G.in[best]) --readers_left[t];
    for (int t : G.out[best]) exists[t] = 1;
  }
  return RAF_OK;
}

extern "C" raf_status raf_remat_plan(const raf_op_graph* graph, int64_t budget_bytes, int32_t* sequence_out,
                                     int32_t sequence_cap, int32_t* sequence_len, int32_t* evicted_tensor,
                                     int32_t* evicted_pos, int32_t evicted_cap, int32_t* n_evicted,
                                     raf_remat_summary* summary) {
  Graph G;
  if (!load_graph(graph, G)) return RAF_EINVAL;
  if (!sequence_len || !n_evicted || !summary || sequence_cap < 0 || evicted_cap < 0) return RAF_EINVAL;
  PlanResult R;
  if (!plan_remat(G, budget_bytes, R)) return RAF_EINVAL;
  *sequence_len = (int32_t)R.seq.size();
  *n_evicted = (int32_t)R.ev_tensor.size();
  summary->peak_before = R.peak_before;
  summary->peak_after = R.peak_after;
  summary->fits = R.fits ? 1 : 0;
  summary->extra_latency = R.extra_latency;
  if ((size_t)sequence_cap < R.seq.size() || (size_t)evicted_cap < R.ev_tensor.size()) return RAF_EWORKSPACE;
  if (!R.seq.empty() && !sequence_out) return RAF_EINVAL;
  if (!R.ev_tensor.empty() && (!evicted_tensor || !evicted_pos)) return RAF_EINVAL;
  std::copy(R.seq.begin(), R.seq.end(), sequence_out);
  std::copy(R.ev_tensor.begin(), R.ev_tensor.end(), evicted_tensor);
  std::copy(R.ev_pos.begin(), R.ev_pos.end(), evicted_pos);
  return RAF_OK;
}

extern "C" raf_status raf_layer_stack_graph(const raf_layer_desc* desc, int32_t layers, const double* replay_us,
                                            raf_op_graph* sizes, int32_t* in_begin, int32_t* in_ids,
                                            int32_t* out_begin, int32_t* out_ids, double* latency, int64_t* bytes,
                                            uint8_t* flags, int32_t* owner_layer, int32_t* owner_bit,
                                            int32_t* n_in_ids, int32_t* n_out_ids) {
  raf_status rc = validate_desc(desc);
  if (rc != RAF_OK) return rc;
  if (layers < 1 || layers > 512 || !sizes || !n_in_ids || !n_out_ids) return RAF_EINVAL;
  StackGraph S;
  if (!build_stack(*desc, layers, replay_us, S)) return RAF_EINVAL;
  sizes->n_ops = (int32_t)S.lat.size();
  sizes->n_tensors = (int32_t)S.bytes.size();
  *n_in_ids = (int32_t)S.in_ids.size();
  *n_out_ids = (int32_t)S.out_ids.size();
  if (!in_begin) return RAF_OK;   // size query
  if (!in_ids || !out_begin || !out_ids || !latency || !bytes || !flags || !owner_layer || !owner_bit) return RAF_EINVAL;
  std::copy(S.in_begin.begin(), S.in_begin.end(), in_begin);
  std::copy(S.in_ids.begin(), S.in_ids.end(), in_ids);
  std::copy(S.out_begin.begin(), S.out_begin.end(), out_begin);
  std::copy(S.out_ids.begin(), S.out_ids.end(), out_ids);
  std::copy(S.lat.begin(), S.lat.end(), latency);
  std::copy(S.bytes.begin(), S.bytes.end(), bytes);
  std::copy(S.flags.begin(), S.flags.end(), flags);
  std::copy(S.owner_layer.begin(), S.owner_layer.end(), owner_layer);
  std::copy(S.owner_bit.begin(), S.owner_bit.end(), owner_bit);
  return RAF_OK;
}

extern "C" raf_status raf_layer_stack_remat(const raf_layer_desc* desc, int32_t layers, int64_t budget_bytes,
                                            const double* replay_us, uint32_t* remat_out, raf_remat_summary* summary) {
  raf_status rc = validate_desc(desc);
  if (rc != RAF_OK) return rc;
  if (layers < 1 || layers > 512 || !remat_out || !summary) return RAF_EINVAL;
  StackGraph S;
  if (!build_stack(*desc, layers, replay_us, S)) return RAF_EINVAL;
  const raf_op_graph g = view(S);
  Graph G;
  if (!load_graph(&g, G)) return RAF_EINVAL;
  PlanResult R;
  if (!plan_remat(G, budget_bytes, R)) return RAF_EINVAL;
  for (int l = 0; l < layers; ++l) remat_out[l] = 0;
  for (int t : R.ev_tensor)
    if (S.owner_layer[t] >= 0) remat_out[S.owner_layer[t]] |= (uint32_t)S.owner_bit[t];
  summary->peak_before = R.peak_before;
  summary->peak_after = R.peak_after;
  summary->fits = R.fits ? 1 : 0;
  summary->extra_latency = R.extra_latency;
  return RAF_OK;
}
