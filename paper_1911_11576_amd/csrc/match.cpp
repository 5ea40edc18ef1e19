// The recogniser: maps a validated fusion group onto one of the hand-written stitched
// schedules, or reports why none applies.  This is what is left of the paper's kernel
// generation loop (Algorithm 3) when every schedule is written ahead of time: instead of
// emitting code per template, the group's dataflow is matched structurally, its
// constants and operand bindings are extracted, and a schedule is selected.  Sums and
// products are flattened before matching, so operand order and association of
// add/subtract/multiply chains do not matter.
#include "match.h"

#include <algorithm>
#include <cmath>

namespace fs {
namespace {

struct Term { int node; int sign; };

struct Rec {
  const Graph& g;
  explicit Rec(const Graph& gr) : g(gr) {}

  bool cst(int n, double* v) const {
    if (g[n].kind != FS_CONSTANT) return false;
    *v = g[n].attr;
    return true;
  }
  // parameter read in its storage dtype, possibly widened by a convert
  int in_param(int n) const {
    if (g[n].kind == FS_CONVERT) n = g[n].operand[0];
    return g[n].kind == FS_PARAMETER ? n : -1;
  }
  int strip_convert(int n) const { return g[n].kind == FS_CONVERT ? g[n].operand[0] : n; }

  // n as a signed sum of terms plus a constant; `stop` (if >= 0) is kept whole as a term
  void sum_terms(int n, int sign, std::vector<Term>& t, double& c, int stop = -1) const {
    const Node& x = g[n];
    double v;
    if (n == stop) t.push_back({n, sign});
    else if (x.kind == FS_ADD) { sum_terms(x.operand[0], sign, t, c, stop); sum_terms(x.operand[1], sign, t, c, stop); }
    else if (x.kind == FS_SUBTRACT) { sum_terms(x.operand[0], sign, t, c, stop); sum_terms(x.operand[1], -sign, t, c, stop); }
    else if (x.kind == FS_NEGATE) sum_terms(x.operand[0], -sign, t, c, stop);
    else if (cst(n, &v)) c += sign * v;
    else t.push_back({n, sign});
  }
  // n == a - broadcast_rows(b): returns true and the two nodes
  bool minus_row_bcast(int n, int* a, int* b) const {
    if (g[n].kind != FS_SUBTRACT) return false;
    *b = row_bcast(g[n].operand[1]);
    *a = g[n].operand[0];
    return *b >= 0;
  }
  void prod_factors(int n, std::vector<int>& f, double& c) const {
    const Node& x = g[n];
    double v;
    if (x.kind == FS_MULTIPLY) { prod_factors(x.operand[0], f, c); prod_factors(x.operand[1], f, c); }
    else if (x.kind == FS_NEGATE) { c = -c; prod_factors(x.operand[0], f, c); }
    else if (x.kind == FS_DIVIDE && cst(x.operand[1], &v)) { c /= v; prod_factors(x.operand[0], f, c); }
    else if (cst(n, &v)) c *= v;
    else f.push_back(n);
  }

  // [R...] -> [R..., C]: operand supplies one value per row
  int row_bcast(int n) const {
    const Node& x = g[n];
    if (x.kind != FS_BROADCAST || x.axis != 0) return -1;
    const Node& a = g[x.operand[0]];
    if (a.rank != x.rank - 1) return -1;
    for (int d = 0; d < a.rank; ++d) if (a.shape[d] != x.shape[d]) return -1;
    return x.operand[0];
  }
  // [C] -> [R..., C]: operand supplies one value per column
  int col_bcast(int n) const {
    const Node& x = g[n];
    if (x.kind != FS_BROADCAST || x.axis != x.rank - 1) return -1;
    const Node& a = g[x.operand[0]];
    if (a.rank != 1 || a.shape[0] != x.shape[x.rank - 1]) return -1;
    return x.operand[0];
  }
  int last_axis_reduce(int n, int kind) const {
    const Node& x = g[n];
    if (x.kind != kind) return -1;
    return x.axis == g[x.operand[0]].rank - 1 ? x.operand[0] : -1;
  }
  // sum over the last axis times 1/N (spelled as divide by N or multiply by 1/N)
  int row_mean(int n) const {
    std::vector<int> f; double c = 1.0;
    prod_factors(n, f, c);
    if (f.size() != 1) return -1;
    const int x = last_axis_reduce(f[0], FS_REDUCE_SUM);
    if (x < 0) return -1;
    const double N = (double)g[x].shape[g[x].rank - 1];
    return std::fabs(c * N - 1.0) < 1e-9 ? x : -1;
  }
};

int64_t leading_rows(const Node& n) {
  int64_t r = 1;
  for (int d = 0; d + 1 < n.rank; ++d) r *= n.shape[d];
  return r;
}

// ---- softmax over the last axis: p = e / sum(e), e = exp(z - max(z)); returns z ----------
int match_softmax_tail(const Rec& r, int p) {
  const Graph& g = r.g;
  if (g[p].kind != FS_DIVIDE) return -1;
  const int e = g[p].operand[0];
  const int den = r.row_bcast(g[p].operand[1]);
  if (den < 0 || r.last_axis_reduce(den, FS_REDUCE_SUM) != e) return -1;
  if (g[e].kind != FS_EXP) return -1;
  int z = -1, zmax = -1;
  if (!r.minus_row_bcast(g[e].operand[0], &z, &zmax)) return -1;
  if (r.last_axis_reduce(zmax, FS_REDUCE_MAX) != z) return -1;
  return z;
}

// ---- LayerNorm over the last axis --------------------------------------------------------
struct LnTail { int r = -1, gamma = -1, beta = -1; double eps = 0; };

bool match_layernorm_tail(const Rec& r, int y, LnTail* out) {
  const Graph& g = r.g;
  std::vector<Term> t; double c = 0;
  r.sum_terms(y, +1, t, c);
  if (c != 0) return false;
  int core = -1;
  if (t.size() == 1 && t[0].sign > 0) core = t[0].node;
  else if (t.size() == 2 && t[0].sign > 0 && t[1].sign > 0) {
    for (int k = 0; k < 2; ++k) {
      const int b = r.col_bcast(t[k].node);
      if (b >= 0 && r.in_param(b) >= 0) { out->beta = r.in_param(b); core = t[1 - k].node; break; }
    }
  }
  if (core < 0) return false;
  std::vector<int> f; double pc = 1;
  r.prod_factors(core, f, pc);
  if (pc != 1.0) return false;
  int rstd = -1, cn = -1;
  for (int n : f) {
    const int rb = r.row_bcast(n), cb = r.col_bcast(n);
    if (rb >= 0 && g[rb].kind == FS_RSQRT && rstd < 0) rstd = rb;
    else if (cb >= 0 && r.in_param(cb) >= 0 && out->gamma < 0) out->gamma = r.in_param(cb);
    else if (cn < 0) cn = n;
    else return false;
  }
  if (rstd < 0 || cn < 0) return false;
  // cn = r - mean(r)
  int rr = -1, mean = -1;
  if (!r.minus_row_bcast(cn, &rr, &mean) || r.row_mean(mean) != rr) return false;
  out->r = rr;
  // rstd = rsqrt(mean(cn*cn) + eps)
  t.clear(); c = 0;
  r.sum_terms(g[rstd].operand[0], +1, t, c);
  if (t.size() != 1 || t[0].sign != +1 || !(c >= 0)) return false;
  out->eps = c;
  const int sq = r.row_mean(t[0].node);
  if (sq < 0) return false;
  f.clear(); pc = 1;
  r.prod_factors(sq, f, pc);
  return pc == 1.0 && f.size() == 2 && f[0] == cn && f[1] == cn;
}

// gel = c_half*h*(1 + tanh(k0*(h + k1*h^3))), in any association and operand order
bool match_gelu_core(const Rec& r, int gel, int* h_out, double* c_half, double* k0_out, double* k1_out) {
  const Graph& g = r.g;
  std::vector<int> f; double ch = 1;
  r.prod_factors(gel, f, ch);
  if (f.size() != 2) return false;
  int h = -1, th = -1;
  for (int k = 0; k < 2 && th < 0; ++k) {
    std::vector<Term> tt; double one = 0;
    r.sum_terms(f[k], +1, tt, one);
    if (one == 1.0 && tt.size() == 1 && tt[0].sign > 0 && g[tt[0].node].kind == FS_TANH) { th = tt[0].node; h = f[1 - k]; }
  }
  if (th < 0) return false;
  std::vector<int> uf; double k0 = 1;
  r.prod_factors(g[th].operand[0], uf, k0);
  if (uf.size() != 1) return false;
  std::vector<Term> wt; double wc = 0;
  r.sum_terms(uf[0], +1, wt, wc, h);
  if (wc != 0 || wt.size() != 2 || wt[0].sign < 0 || wt[1].sign < 0) return false;
  if (wt[0].node != h) std::swap(wt[0], wt[1]);
  if (wt[0].node != h) return false;
  std::vector<int> qf; double k1 = 1;
  r.prod_factors(wt[1].node, qf, k1);
  if (qf.size() != 3 || qf[0] != h || qf[1] != h || qf[2] != h) return false;
  *h_out = h; *c_half = ch; *k0_out = k0; *k1_out = k1;
  return true;
}

// r = gel [+ residual], h = x [+ bias]
bool match_gelu_prologue(const Rec& r, int rn, RowSpec* sp, int* x_node, int* bias_node, int* res_node) {
  const Graph& g = r.g;
  std::vector<Term> t; double c = 0;
  r.sum_terms(rn, +1, t, c);
  if (c != 0) return false;
  int gel = -1;
  *res_node = -1;
  if (t.size() == 1 && t[0].sign > 0) gel = t[0].node;
  else if (t.size() == 2 && t[0].sign > 0 && t[1].sign > 0) {
    for (int k = 0; k < 2; ++k) {
      const int p = r.in_param(t[k].node);
      if (p >= 0 && g[p].same_shape(g[rn])) { *res_node = p; gel = t[1 - k].node; break; }
    }
  }
  if (gel < 0) return false;
  int h = -1;
  double ch = 1, k0 = 1, k1 = 1;
  if (!match_gelu_core(r, gel, &h, &ch, &k0, &k1)) return false;
  // h = x (+ bias)
  *bias_node = -1;
  int xp = r.in_param(h);
  if (xp < 0) {
    std::vector<Term> ht; double hc = 0;
    r.sum_terms(h, +1, ht, hc);
    if (hc != 0 || ht.size() != 2 || ht[0].sign < 0 || ht[1].sign < 0) return false;
    for (int k = 0; k < 2; ++k) {
      const int cb = r.col_bcast(ht[k].node);
      if (cb >= 0 && r.in_param(cb) >= 0) { *bias_node = r.in_param(cb); xp = r.in_param(ht[1 - k].node); break; }
    }
    if (xp < 0 || *bias_node < 0) return false;
  }
  if (!g[xp].same_shape(g[rn])) return false;
  *x_node = xp;
  sp->gelu = true;
  sp->gelu_half = (float)ch; sp->gelu_k0 = (float)k0; sp->gelu_k1 = (float)k1;
  return true;
}

bool same_dtype_params(const Graph& g, int dt, std::initializer_list<int> nodes) {
  for (int n : nodes) if (n >= 0 && g[n].dtype != dt) return false;
  return true;
}

bool try_row_layernorm(const Rec& r, Match* m) {
  const Graph& g = r.g;
  if (g.outputs.size() != 1) return false;
  const Node& out = g[g.outputs[0]];
  if (out.rank < 2) return false;
  LnTail ln;
  if (!match_layernorm_tail(r, r.strip_convert(out.operand[0]), &ln)) return false;
  RowSpec sp;
  sp.core = CORE_LAYERNORM;
  sp.cols = out.shape[out.rank - 1];
  sp.rows = leading_rows(out);
  sp.dtype = out.dtype;
  sp.eps = (float)ln.eps;
  int x = r.in_param(ln.r), bias = -1, res = -1;
  if (x < 0 && !match_gelu_prologue(r, ln.r, &sp, &x, &bias, &res)) return false;
  if (!g[x].same_shape(out)) return false;
  if (!same_dtype_params(g, sp.dtype, {x, bias, res, ln.gamma, ln.beta})) {
    m->why = "row schedule: parameters and output must share one storage dtype";
    return false;
  }
  sp.in_x = g[x].ordinal;
  sp.in_bias = bias >= 0 ? g[bias].ordinal : -1;
  sp.in_res = res >= 0 ? g[res].ordinal : -1;
  sp.in_gamma = ln.gamma >= 0 ? g[ln.gamma].ordinal : -1;
  sp.in_beta = ln.beta >= 0 ? g[ln.beta].ordinal : -1;
  m->kind = MATCH_ROW;
  m->row = sp;
  return true;
}

bool try_row_softmax(const Rec& r, Match* m) {
  const Graph& g = r.g;
  if (g.outputs.size() != 1) return false;
  const Node& out = g[g.outputs[0]];
  if (out.rank < 2) return false;
  const int z = match_softmax_tail(r, r.strip_convert(out.operand[0]));
  if (z < 0) return false;
  std::vector<Term> t; double c = 0;
  r.sum_terms(z, +1, t, c);
  if (c != 0 || t.empty() || t.size() > 2) return false;
  for (const Term& x : t) if (x.sign < 0) return false;
  RowSpec sp;
  sp.core = CORE_SOFTMAX;
  sp.cols = out.shape[out.rank - 1];
  sp.rows = leading_rows(out);
  sp.dtype = out.dtype;
  // which term is scale*scores: the one that is a product with a full-shape parameter
  int s_node = -1, m_term = -1;
  for (size_t k = 0; k < t.size() && s_node < 0; ++k) {
    std::vector<int> f; double sc = 1;
    r.prod_factors(t[k].node, f, sc);
    if (f.size() == 1 && r.in_param(f[0]) >= 0 && g[r.in_param(f[0])].same_shape(out)) {
      s_node = r.in_param(f[0]);
      sp.scale = (float)sc;
      if (t.size() == 2) m_term = t[1 - k].node;
    }
  }
  if (s_node < 0) return false;
  int mask = -1;
  if (m_term >= 0) {
    mask = r.in_param(m_term);
    if (mask >= 0) {
      if (!g[mask].same_shape(out)) return false;
    } else {
      const Node& b = g[m_term];
      if (b.kind != FS_BROADCAST || b.axis != 0) return false;
      mask = r.in_param(b.operand[0]);
      if (mask < 0) return false;
      const Node& mk = g[mask];
      if (mk.rank != out.rank || mk.shape[mk.rank - 1] != sp.cols) return false;
      // leading dims collapse to (d0, d1, d2) right-aligned; the mask's strides are 0 where
      // it is expanded
      int64_t d[3] = {1, 1, 1}, e[3] = {1, 1, 1};
      for (int k = 0; k + 1 < out.rank; ++k) { d[3 - (out.rank - 1) + k] = out.shape[k]; e[3 - (out.rank - 1) + k] = mk.shape[k]; }
      bool full = true;
      for (int k = 0; k < 3; ++k) full = full && d[k] == e[k];
      if (!full) {
        sp.mask_d1 = d[1]; sp.mask_d2 = d[2];
        sp.mask_stride[0] = e[0] > 1 ? e[1] * e[2] : 0;
        sp.mask_stride[1] = e[1] > 1 ? e[2] : 0;
        sp.mask_stride[2] = e[2] > 1 ? 1 : 0;
      }
    }
  }
  if (!same_dtype_params(g, sp.dtype, {s_node, mask})) {
    m->why = "row schedule: parameters and output must share one storage dtype";
    return false;
  }
  sp.in_x = g[s_node].ordinal;
  sp.in_mask = mask >= 0 ? g[mask].ordinal : -1;
  m->kind = MATCH_ROW;
  m->row = sp;
  return true;
}

// ---- LayerNorm backward ------------------------------------------------------------------
struct Factors {
  int dy = -1, gamma = -1, x = -1, mean = -1, rstd = -1, rowb = -1, other = -1;
  int count = 0;
  bool clean = true;   // constant factor 1, no class seen twice
};

Factors classify(const Rec& r, int n, int rank2_rows_cols_of) {
  const Graph& g = r.g;
  Factors out;
  std::vector<int> f; double c = 1;
  r.prod_factors(n, f, c);
  if (c != 1.0) out.clean = false;
  const Node& ref = g[rank2_rows_cols_of];
  for (int k : f) {
    ++out.count;
    const int p = r.in_param(k), rb = r.row_bcast(k), cb = r.col_bcast(k);
    if (p >= 0 && g[p].same_shape(ref)) { if (out.dy >= 0) out.clean = false; out.dy = p; continue; }
    if (cb >= 0 && r.in_param(cb) >= 0) { if (out.gamma >= 0) out.clean = false; out.gamma = r.in_param(cb); continue; }
    if (rb >= 0 && r.in_param(rb) >= 0) { if (out.rstd >= 0) out.clean = false; out.rstd = r.in_param(rb); continue; }
    if (rb >= 0) { if (out.rowb >= 0) out.clean = false; out.rowb = rb; continue; }
    std::vector<Term> t; double sc = 0;
    r.sum_terms(k, +1, t, sc);
    if (sc == 0 && t.size() == 2) {
      if (t[0].sign < 0) std::swap(t[0], t[1]);
      const int xp = r.in_param(t[0].node);
      const int mb = t[1].sign < 0 ? r.row_bcast(t[1].node) : -1;
      if (t[0].sign > 0 && xp >= 0 && g[xp].same_shape(ref) && mb >= 0 && r.in_param(mb) >= 0) {
        if (out.x >= 0) out.clean = false;
        out.x = xp; out.mean = r.in_param(mb);
        continue;
      }
    }
    if (out.other >= 0) out.clean = false;
    out.other = k;
  }
  return out;
}

bool try_layernorm_bwd(const Rec& r, Match* m) {
  const Graph& g = r.g;
  if (g.outputs.empty() || g.outputs.size() > 3) return false;
  LnBwdSpec sp;
  int dy = -1, x = -1, mean = -1, rstd = -1, gamma = -1;
  auto bind = [](int* slot, int v) { if (*slot < 0) *slot = v; return *slot == v; };
  // find the [R,C] reference shape: the first rank-2 parameter
  int ref = -1;
  for (int p : g.params) if (g[p].rank == 2) { ref = p; break; }
  if (ref < 0) return false;
  for (int o : g.outputs) {
    const Node& out = g[o];
    const int v = out.operand[0];
    if (out.dtype != FS_F32) return false;
    if (out.rank == 1) {
      if (g[v].kind != FS_REDUCE_SUM || g[v].axis != 0 || g[g[v].operand[0]].rank != 2) return false;
      const Factors f = classify(r, g[v].operand[0], ref);
      if (!f.clean) return false;
      if (f.count == 1 && f.dy >= 0) {                       // dbeta = sum_i dy
        if (sp.out_dbeta >= 0 || !bind(&dy, f.dy)) return false;
        sp.out_dbeta = out.ordinal;
      } else if (f.count == 3 && f.dy >= 0 && f.x >= 0 && f.rstd >= 0) {   // dgamma = sum_i dy*xhat
        if (sp.out_dgamma >= 0 || !bind(&dy, f.dy) || !bind(&x, f.x) || !bind(&mean, f.mean) || !bind(&rstd, f.rstd)) return false;
        sp.out_dgamma = out.ordinal;
      } else return false;
    } else if (out.rank == 2) {
      if (sp.out_dx >= 0) return false;
      const Factors f = classify(r, v, ref);                  // dx = w * rstd
      if (!f.clean || f.count != 2 || f.rstd < 0 || f.other < 0 || !bind(&rstd, f.rstd)) return false;
      std::vector<Term> t; double c = 0;
      r.sum_terms(f.other, +1, t, c);
      if (c != 0 || t.size() != 3) return false;
      int seen = 0;
      for (const Term& tm : t) {
        const int rb = r.row_bcast(tm.node);
        if (tm.sign > 0) {                                    // + dy*gamma
          const Factors a = classify(r, tm.node, ref);
          if (!a.clean || a.count != 2 || a.dy < 0 || a.gamma < 0 || !bind(&dy, a.dy) || !bind(&gamma, a.gamma)) return false;
          seen |= 1;
        } else if (rb >= 0) {                                 // - mean_j(dy*gamma)
          const int inner = r.row_mean(rb);
          if (inner < 0) return false;
          const Factors a = classify(r, inner, ref);
          if (!a.clean || a.count != 2 || a.dy < 0 || a.gamma < 0 || !bind(&dy, a.dy) || !bind(&gamma, a.gamma)) return false;
          seen |= 2;
        } else {                                              // - xhat * mean_j(dy*gamma*xhat)
          const Factors a = classify(r, tm.node, ref);
          if (!a.clean || a.count != 3 || a.x < 0 || a.rstd < 0 || a.rowb < 0) return false;
          if (!bind(&x, a.x) || !bind(&mean, a.mean) || !bind(&rstd, a.rstd)) return false;
          const int inner = r.row_mean(a.rowb);
          if (inner < 0) return false;
          const Factors b = classify(r, inner, ref);
          if (!b.clean || b.count != 4 || b.dy < 0 || b.gamma < 0 || b.x < 0 || b.rstd < 0) return false;
          if (!bind(&dy, b.dy) || !bind(&gamma, b.gamma) || !bind(&x, b.x) || !bind(&mean, b.mean) || !bind(&rstd, b.rstd)) return false;
          seen |= 4;
        }
      }
      if (seen != 7) return false;
      sp.out_dx = out.ordinal;
    } else return false;
  }
  if (dy < 0) return false;
  const Node& d = g[dy];
  if (d.dtype != FS_F32) { m->why = "LayerNorm-backward schedule is fp32 only"; return false; }
  for (int p : {x, gamma, mean, rstd}) if (p >= 0 && g[p].dtype != FS_F32) { m->why = "LayerNorm-backward schedule is fp32 only"; return false; }
  if (x >= 0 && (g[mean].rank != 1 || g[rstd].rank != 1)) return false;
  sp.rows = d.shape[0]; sp.cols = d.shape[1];
  sp.in_dy = d.ordinal;
  sp.in_x = x >= 0 ? g[x].ordinal : -1;
  sp.in_gamma = gamma >= 0 ? g[gamma].ordinal : -1;
  sp.in_mean = mean >= 0 ? g[mean].ordinal : -1;
  sp.in_rstd = rstd >= 0 ? g[rstd].ordinal : -1;
  m->kind = MATCH_LNBWD;
  m->lnbwd = sp;
  return true;
}

// ---- batched dot -> softmax -> batched dot, with the elementwise ops around them ---------------
// softmax over the last axis with the nodes a second output may refer to: z, max(z), sum(exp(z - max))
struct SoftmaxParts { int z = -1, zmax = -1, den = -1; };
bool match_softmax_parts(const Rec& r, int p, SoftmaxParts* out) {
  const Graph& g = r.g;
  if (g[p].kind != FS_DIVIDE) return false;
  const int e = g[p].operand[0];
  const int den = r.row_bcast(g[p].operand[1]);
  if (den < 0 || r.last_axis_reduce(den, FS_REDUCE_SUM) != e) return false;
  if (g[e].kind != FS_EXP) return false;
  int z = -1, zmax = -1;
  if (!r.minus_row_bcast(g[e].operand[0], &z, &zmax)) return false;
  if (r.last_axis_reduce(zmax, FS_REDUCE_MAX) != z) return false;
  out->z = z; out->zmax = zmax; out->den = den;
  return true;
}

bool try_attention(const Rec& r, Match* m) {
  const Graph& g = r.g;
  if (g.outputs.empty() || g.outputs.size() > 2) return false;
  AttnSpec sp;
  int o_out = -1, lse_out = -1;
  for (int oi : g.outputs) {
    if (g[oi].rank == 3 && o_out < 0) o_out = oi;
    else if (g[oi].rank == 2 && lse_out < 0) lse_out = oi;
    else return false;
  }
  if (o_out < 0) return false;
  const Node& out = g[o_out];
  // ---- epilogue: out = convert(dot * gate + res), gate and residual optional, parameters of o's shape and dtype
  int top = r.strip_convert(out.operand[0]);
  std::vector<Term> ot; double oc = 0;
  r.sum_terms(top, +1, ot, oc);
  if (oc != 0 || ot.empty() || ot.size() > 2) return false;
  int core = -1, res = -1;
  if (ot.size() == 1) {
    if (ot[0].sign < 0) return false;
    core = ot[0].node;
  } else {
    for (int k = 0; k < 2 && res < 0; ++k) {
      const int pr = r.in_param(ot[k].node);
      if (pr >= 0 && ot[k].sign > 0 && ot[1 - k].sign > 0) { res = pr; core = ot[1 - k].node; }
    }
    if (res < 0) return false;
  }
  std::vector<int> of; double ofc = 1;
  r.prod_factors(core, of, ofc);
  if (ofc != 1.0 || of.empty() || of.size() > 2) return false;
  int o = -1, gate = -1;
  for (int n : of) {
    if (g[n].kind == FS_DOT && o < 0) o = n;
    else if (r.in_param(n) >= 0 && gate < 0) gate = r.in_param(n);
    else return false;
  }
  if (o < 0 || g[o].axis != 0) return false;
  const int v = g[o].operand[1];
  if (g[v].kind != FS_PARAMETER) return false;
  const int p = r.strip_convert(g[o].operand[0]);
  SoftmaxParts sm;
  if (!match_softmax_parts(r, p, &sm)) return false;
  // ---- second output: max(z) + log(sum(exp(z - max(z)))), one value per score row
  if (lse_out >= 0) {
    std::vector<Term> lt; double lc = 0;
    r.sum_terms(g[lse_out].operand[0], +1, lt, lc);
    if (lc != 0 || lt.size() != 2 || lt[0].sign < 0 || lt[1].sign < 0) return false;
    bool ok = false;
    for (int k = 0; k < 2; ++k)
      if (lt[k].node == sm.zmax && g[lt[1 - k].node].kind == FS_LOG && g[lt[1 - k].node].operand[0] == sm.den) ok = true;
    if (!ok) return false;
    if (g[lse_out].dtype != FS_F32) { m->why = "attention schedule: the log-sum-exp output must be f32"; return false; }
  }
  // ---- z: the first dot under, from the outside in, any of: a positive constant factor, one additive
  // fp32 mask or bias (a parameter, possibly broadcast over the batch or the query rows), a causal mask.
  // What sits outside the causal mask is applied to the fill value too, which only -inf survives unchanged.
  double scale = 1.0;
  int mask = -1;           // the parameter
  int64_t mask_sb = 0, mask_sq = 0;
  bool outside = false;    // something was peeled that the causal fill would pass through
  int n = sm.z;
  const Node& zs = g[sm.z];
  if (zs.rank != 3) return false;
  const int64_t SQ = zs.shape[1], SK = zs.shape[2];
  for (int guard = 0; guard < 8 && g[n].kind != FS_DOT; ++guard) {
    const Node& x = g[n];
    if (x.kind == FS_CAUSAL_MASK) {
      if (sp.causal) return false;
      sp.causal = true;
      sp.fill = (float)x.attr;
      if (outside && !(sp.fill == -INFINITY && scale > 0)) {
        m->why = "attention schedule: a scale or mask applied after the causal mask needs fill=-inf and scale>0";
        return false;
      }
      n = x.operand[0];
      continue;
    }
    if (x.kind == FS_ADD) {
      if (mask >= 0 || scale != 1.0) return false;      // one mask, and not inside the scale
      int found = -1;
      for (int k = 0; k < 2 && found < 0; ++k) {
        const int t = x.operand[k];
        int src = -1;
        int64_t sb = 0, sq = 0;
        if (g[t].kind == FS_PARAMETER && g[t].rank == 3) { src = t; sb = SQ * SK; sq = SK; }
        else if (g[t].kind == FS_BROADCAST && g[g[t].operand[0]].kind == FS_PARAMETER) {
          const Node& pm = g[g[t].operand[0]];
          const int ax = g[t].axis;
          // operand dim d sits at result dim ax + d; extent-1 dims are expanded
          int64_t ext[3] = {1, 1, 1};
          bool fits = ax >= 0 && ax + pm.rank <= 3;
          for (int d = 0; fits && d < pm.rank; ++d) ext[ax + d] = pm.shape[d];
          if (fits && ext[2] == SK && (ext[1] == SQ || ext[1] == 1) && (ext[0] == zs.shape[0] || ext[0] == 1)) {
            src = g[t].operand[0];
            sq = ext[1] == 1 ? 0 : SK;
            sb = ext[0] == 1 ? 0 : ext[1] * SK;
          }
        }
        if (src >= 0 && g[src].dtype == FS_F32) { found = k; mask = src; mask_sb = sb; mask_sq = sq; }
      }
      if (found < 0) return false;
      outside = true;
      n = x.operand[1 - found];
      continue;
    }
    // a constant factor
    std::vector<int> f; double c = 1;
    r.prod_factors(n, f, c);
    if (f.size() != 1 || f[0] == n) return false;
    scale *= c;
    outside = true;
    n = f[0];
  }
  if (g[n].kind != FS_DOT || g[n].axis != 1) return false;
  const int q = g[n].operand[0], k = g[n].operand[1];
  if (g[q].kind != FS_PARAMETER || g[k].kind != FS_PARAMETER) return false;
  const int dt = g[q].dtype;
  if (dt == FS_F32) { m->why = "attention schedule: fp32 operands have no MFMA path here (use f16 or bf16)"; return false; }
  if (g[k].dtype != dt || g[v].dtype != dt || out.dtype != dt) { m->why = "attention schedule: q, k, v and o must share one 16-bit dtype"; return false; }
  if (g[g[o].operand[0]].dtype != dt) return false;
  if (g[n].dtype != FS_F32 || g[o].dtype != FS_F32) { m->why = "attention schedule: both dots must accumulate in f32"; return false; }
  sp.batch = g[q].shape[0]; sp.sq = g[q].shape[1]; sp.dim = g[q].shape[2]; sp.sk = g[k].shape[1];
  if (g[v].shape[1] != sp.sk || g[v].shape[2] != sp.dim) {
    m->why = "attention schedule: needs equal key/value lengths and equal q/v head dims";
    return false;
  }
  for (int e : {gate, res}) {
    if (e < 0) continue;
    if (g[e].dtype != dt || g[e].rank != 3 || !g[e].same_shape(out)) {
      m->why = "attention schedule: gate and residual must have the output's shape and dtype";
      return false;
    }
  }
  sp.dtype = dt;
  sp.scale = (float)scale;
  sp.in_q = g[q].ordinal; sp.in_k = g[k].ordinal; sp.in_v = g[v].ordinal;
  sp.in_mask = mask >= 0 ? g[mask].ordinal : -1;
  sp.mask_sb = mask_sb; sp.mask_sq = mask_sq;
  sp.in_gate = gate >= 0 ? g[gate].ordinal : -1;
  sp.in_res = res >= 0 ? g[res].ordinal : -1;
  sp.out_o = out.ordinal;
  sp.out_lse = lse_out >= 0 ? g[lse_out].ordinal : -1;
  m->kind = MATCH_ATTN;
  m->attn = sp;
  return true;
}

}  // namespace

std::vector<GeluIdiom> find_gelu_idioms(const Graph& g) {
  std::vector<GeluIdiom> found;
  const int n = g.size();
  Rec r(g);
  auto n_operands = [&](const Node& x) {
    switch (x.kind) {
      case FS_PARAMETER: case FS_CONSTANT: return 0;
      case FS_ADD: case FS_SUBTRACT: case FS_MULTIPLY: case FS_DIVIDE: case FS_MAXIMUM: case FS_DOT: return 2;
      default: return 1;
    }
  };
  std::vector<std::vector<int>> users(n);
  for (int i = 0; i < n; ++i)
    for (int j = 0; j < n_operands(g[i]); ++j) users[g[i].operand[j]].push_back(i);
  std::vector<char> taken(n, 0);
  for (int i = n - 1; i >= 0; --i) {
    if (g[i].kind != FS_MULTIPLY || taken[i]) continue;
    GeluIdiom id;
    if (!match_gelu_core(r, i, &id.h, &id.half, &id.k0, &id.k1)) continue;
    // the ops between h and the result (constants aside)
    std::vector<int> stack{i};
    std::vector<char> seen(n, 0);
    bool ok = true;
    while (!stack.empty() && ok) {
      const int v = stack.back(); stack.pop_back();
      for (int j = 0; j < n_operands(g[v]); ++j) {
        const int o = g[v].operand[j];
        if (o == id.h || g[o].kind == FS_CONSTANT || seen[o]) continue;
        const int k = g[o].kind;
        if (!(k == FS_MULTIPLY || k == FS_ADD || k == FS_SUBTRACT || k == FS_NEGATE || k == FS_TANH || k == FS_DIVIDE)) { ok = false; break; }
        seen[o] = 1;
        id.interior.push_back(o);
        stack.push_back(o);
      }
    }
    if (!ok) continue;
    // nothing outside the idiom reads an interior value, and none of them is taken already
    seen[i] = 1;
    for (int v : id.interior) {
      if (taken[v]) ok = false;
      for (int u : users[v]) if (!seen[u]) ok = false;
    }
    if (!ok) continue;
    id.out = i;
    for (int v : id.interior) taken[v] = 1;
    taken[i] = 1;
    found.push_back(id);
  }
  return found;
}

bool recognise(const Graph& g, Match* m) {
  Rec r(g);
  m->kind = MATCH_NONE;
  m->why.clear();
  if (try_row_layernorm(r, m)) return true;
  if (try_row_softmax(r, m)) return true;
  if (try_layernorm_bwd(r, m)) return true;
  if (try_attention(r, m)) return true;
  if (m->why.empty()) m->why = "no stitched schedule matches this group";
  m->kind = MATCH_NONE;
  return false;
}

}  // namespace fs
