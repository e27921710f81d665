// Index-map composer and simplifier (paper Sec. 3.2.1).
//
// A map is the source element offset written as an affine combination of
// "atoms": view variables, and // and % of affine arguments.  All coefficients
// and constants are non-negative, every atom has a known range [0, hi], so
// the rewrite rules below are exact on the map's whole domain:
//   (c*Q + R) // c  ->  Q            when 0 <= R < c
//   (c*Q + R) %  c  ->  R            when 0 <= R < c
//   (X // a) // b   ->  X // (a*b)
//   (X % (a*b)) // b -> (X // b) % a
//   (X % a) % b     ->  X % b        when b divides a   (the paper's example)
//   X // c -> 0, X % c -> X          when range(X) < c
//   c*(X // (b*c)) + (X // b) % c -> X // b   (a split followed by the matching merge)
#include "index_map.h"
#include <algorithm>
#include <cstring>

namespace sm {

static int64_t affine_hi(const std::vector<Atom>& atoms, const Affine& a) {
  int64_t h = a.c0;
  for (auto& t : a.terms) h += t.second * atoms[t.first].hi;
  return h;
}

static bool same_affine(const Affine& a, const Affine& b) {
  return a.c0 == b.c0 && a.terms == b.terms;
}

static void add_term(Affine& a, int atom, int64_t coef) {
  if (coef == 0) return;
  for (auto& t : a.terms)
    if (t.first == atom) { t.second += coef; return; }
  a.terms.emplace_back(atom, coef);
  std::sort(a.terms.begin(), a.terms.end());
}

static void add_scaled(Affine& dst, const Affine& src, int64_t s) {
  dst.c0 += s * src.c0;
  for (auto& t : src.terms) add_term(dst, t.first, s * t.second);
}

struct Builder {
  std::vector<Atom>& atoms;
  bool simplify;
  Builder(std::vector<Atom>& a, bool s) : atoms(a), simplify(s) {}

  int intern(const Atom& x) {
    for (size_t i = 0; i < atoms.size(); ++i) {
      const Atom& y = atoms[i];
      if (y.kind == x.kind && y.var == x.var && y.div == x.div && y.mod == x.mod && same_affine(y.arg, x.arg)) return (int)i;
    }
    atoms.push_back(x);
    return (int)atoms.size() - 1;
  }
  Affine var(int v, int64_t extent) {
    if (extent == 1 && simplify) return Affine();     // an index that is always 0
    Atom a; a.kind = ATOM_VAR; a.var = v; a.div = 1; a.mod = 0; a.hi = extent - 1;
    Affine r; r.terms.emplace_back(intern(a), 1);
    return r;
  }
  // (x // b) % a with a == 0 for "no modulus"
  Affine digit(const Affine& x, int64_t b, int64_t a) {
    int64_t h = affine_hi(atoms, x) / b;
    if (simplify) {
      if (a > 0 && h < a) a = 0;                      // modulus never taken
      if (h == 0) return Affine();
      if (b == 1 && a == 0) return x;
    }
    Atom t; t.kind = ATOM_DIGIT; t.var = -1; t.arg = x; t.div = b; t.mod = a;
    t.hi = a > 0 ? std::min(h, a - 1) : h;
    Affine r; r.terms.emplace_back(intern(t), 1);
    return r;
  }
  // c*k*digit(X, b*c, a2) + k*digit(X, b, c)  ->  k*digit(X, b, c*a2): adjacent digits of one value merge
  void recombine(Affine& e) {
    if (!simplify) return;
    bool again = true;
    while (again) {
      again = false;
      for (size_t i = 0; i < e.terms.size() && !again; ++i)
        for (size_t j = 0; j < e.terms.size() && !again; ++j) {
          if (i == j) continue;
          const Atom hiA = atoms[e.terms[i].first], loA = atoms[e.terms[j].first];
          if (hiA.kind != ATOM_DIGIT || loA.kind != ATOM_DIGIT || loA.mod == 0) continue;
          if (!same_affine(hiA.arg, loA.arg)) continue;
          if (hiA.div != loA.div * loA.mod) continue;
          if (e.terms[i].second != e.terms[j].second * loA.mod) continue;
          int64_t k = e.terms[j].second;
          size_t a = std::max(i, j), b = std::min(i, j);
          e.terms.erase(e.terms.begin() + a);
          e.terms.erase(e.terms.begin() + b);
          add_scaled(e, digit(loA.arg, loA.div, hiA.mod ? hiA.mod * loA.mod : 0), k);
          again = true;
        }
    }
  }
  // x = g*y + small with g | c, g > 1 and 0 <= small < g
  bool split_by_factor(const Affine& x, int64_t c, int64_t* g_out, Affine* y, Affine* small) {
    for (auto& cand : x.terms) {
      const int64_t g = cand.second;
      if (g <= 1 || c % g != 0 || g == c) continue;
      Affine yy, ss;
      yy.c0 = x.c0 / g; ss.c0 = x.c0 % g;
      for (auto& t : x.terms) {
        if (t.second % g == 0) add_term(yy, t.first, t.second / g);
        else add_term(ss, t.first, t.second);
      }
      if (ss.terms.empty() && ss.c0 == 0) continue;     // nothing small: plain common factor, handled elsewhere
      if (affine_hi(atoms, ss) < g) { *g_out = g; *y = yy; *small = ss; return true; }
    }
    return false;
  }
  Affine div(Affine x, int64_t c) {
    if (c == 1) return x;
    if (!simplify) return digit(x, c, 0);
    recombine(x);
    Affine q, r;
    q.c0 = x.c0 / c; r.c0 = x.c0 % c;
    for (auto& t : x.terms) {
      if (t.second % c == 0) add_term(q, t.first, t.second / c);
      else add_term(r, t.first, t.second);
    }
    if (affine_hi(atoms, r) < c) return q;
    {  // (g*Y + S) // (g*c') -> Y // c' when 0 <= S < g
      Affine y, sm_;
      int64_t g;
      if (split_by_factor(r, c, &g, &y, &sm_)) {
        add_scaled(q, div(y, c / g), 1);
        recombine(q);
        return q;
      }
    }
    if (r.c0 == 0 && r.terms.size() == 1 && r.terms[0].second == 1) {
      const Atom in = atoms[r.terms[0].first];
      if (in.kind == ATOM_DIGIT && (in.mod == 0 || in.mod % c == 0)) {
        // (X // b) // c -> X // (b*c);  ((X // b) % (c*a)) // c -> (X // (b*c)) % a
        add_scaled(q, digit(in.arg, in.div * c, in.mod ? in.mod / c : 0), 1);
        recombine(q);
        return q;
      }
    }
    add_scaled(q, digit(r, c, 0), 1);
    recombine(q);
    return q;
  }
  Affine mod(Affine x, int64_t c) {
    if (c == 1) return Affine();
    if (!simplify) return digit(x, 1, c);
    recombine(x);
    Affine r;
    r.c0 = x.c0 % c;
    for (auto& t : x.terms) add_term(r, t.first, t.second % c);
    if (affine_hi(atoms, r) < c) return r;
    {  // (g*Y + S) % (g*c') -> g*(Y % c') + S when 0 <= S < g
      Affine y, sm_;
      int64_t g;
      if (split_by_factor(r, c, &g, &y, &sm_)) {
        Affine out = sm_;
        add_scaled(out, mod(y, c / g), g);
        recombine(out);
        return out;
      }
    }
    if (r.c0 == 0 && r.terms.size() == 1 && r.terms[0].second == 1) {
      const Atom in = atoms[r.terms[0].first];
      // (X % a) % c -> X % c when c divides a (the rule printed in Sec. 3.2.1), also through a division
      if (in.kind == ATOM_DIGIT && (in.mod == 0 || in.mod % c == 0)) return digit(in.arg, in.div, c);
    }
    return digit(r, 1, c);
  }
};

// Rebuild expression `e` (over old atoms) with view variables replaced by subst[].
static Affine rebuild(const std::vector<Atom>& old_atoms, const Affine& e, const std::vector<Affine>& subst,
                      Builder& b, std::vector<int>& done, std::vector<Affine>& memo) {
  Affine out; out.c0 = e.c0;
  for (auto& t : e.terms) {
    int id = t.first;
    if (!done[id]) {
      const Atom& a = old_atoms[id];
      if (a.kind == ATOM_VAR) memo[id] = subst[a.var];
      else {
        Affine arg = rebuild(old_atoms, a.arg, subst, b, done, memo);
        memo[id] = a.mod ? b.mod(b.div(arg, a.div), a.mod) : b.div(arg, a.div);
      }
      done[id] = 1;
    }
    add_scaled(out, memo[id], t.second);
  }
  b.recombine(out);
  return out;
}

static void prune(sm_map* m) {   // drop atoms not reachable from the offset expression
  std::vector<int> used(m->atoms.size(), 0);
  std::vector<int> stack;
  for (auto& t : m->offset.terms) stack.push_back(t.first);
  while (!stack.empty()) {
    int id = stack.back(); stack.pop_back();
    if (used[id]) continue;
    used[id] = 1;
    for (auto& t : m->atoms[id].arg.terms) stack.push_back(t.first);
  }
  std::vector<int> remap(m->atoms.size(), -1);
  std::vector<Atom> kept;
  for (size_t i = 0; i < m->atoms.size(); ++i)
    if (used[i]) { remap[i] = (int)kept.size(); kept.push_back(m->atoms[i]); }
  for (auto& a : kept) for (auto& t : a.arg.terms) t.first = remap[t.first];
  for (auto& t : m->offset.terms) t.first = remap[t.first];
  std::sort(m->offset.terms.begin(), m->offset.terms.end());
  for (auto& a : kept) std::sort(a.arg.terms.begin(), a.arg.terms.end());
  m->atoms.swap(kept);
}

// Apply one view operator to (shape, atoms, offset).  Returns false on a bad operator.
static bool apply_view(std::vector<int64_t>& shape, std::vector<Atom>& atoms, Affine& offset,
                       const sm_view_op& op, bool simplify, int* n_made, std::string* err) {
  std::vector<Atom> fresh;
  Builder b(fresh, simplify);
  std::vector<int64_t> nshape;
  std::vector<Affine> subst(shape.size());
  const int rank = (int)shape.size();
  switch (op.kind) {
    case SM_VIEW_PERMUTE: {
      if (op.n != rank) { *err = "permute: rank mismatch"; return false; }
      std::vector<int> seen(rank, 0);
      nshape.resize(rank);
      for (int k = 0; k < rank; ++k) {
        int64_t p = op.arg[k];
        if (p < 0 || p >= rank || seen[p]) { *err = "permute: not a permutation"; return false; }
        seen[p] = 1; nshape[k] = shape[p];
      }
      for (int k = 0; k < rank; ++k) subst[op.arg[k]] = b.var(k, nshape[k]);
      break;
    }
    case SM_VIEW_ROLL: {
      int64_t axis = op.arg[0], r = op.arg[1];
      if (axis < 0 || axis >= rank) { *err = "roll: bad axis"; return false; }
      nshape = shape;
      for (int k = 0; k < rank; ++k) subst[k] = b.var(k, shape[k]);
      int64_t n = shape[axis];
      int64_t add = ((-r) % n + n) % n;               // out[i] = in[(i - r) mod n]
      if (add) { Affine a = subst[axis]; a.c0 += add; subst[axis] = b.mod(a, n); }
      break;
    }
    case SM_VIEW_SLICE: {
      int64_t axis = op.arg[0], start = op.arg[1], stop = op.arg[2], step = op.arg[3] ? op.arg[3] : 1;
      if (axis < 0 || axis >= rank || step < 1 || start < 0 || stop > shape[axis] || start >= stop) {
        *err = "slice: bad arguments"; return false;
      }
      nshape = shape;
      nshape[axis] = (stop - start + step - 1) / step;
      for (int k = 0; k < rank; ++k) subst[k] = b.var(k, nshape[k]);
      Affine a; a.c0 = start; add_scaled(a, subst[axis], step);
      subst[axis] = a;
      break;
    }
    case SM_VIEW_RESHAPE: {
      if (op.n < 1 || op.n > SM_MAX_RANK) { *err = "reshape: bad rank"; return false; }
      int64_t n_old = 1, n_new = 1;
      for (auto s : shape) n_old *= s;
      nshape.assign(op.arg, op.arg + op.n);
      for (auto s : nshape) { if (s < 1) { *err = "reshape: bad extent"; return false; } n_new *= s; }
      if (n_old != n_new) { *err = "reshape: element count differs"; return false; }
      Affine lin;                                      // merge: linear index of the new view
      int64_t st = 1;
      for (int k = op.n - 1; k >= 0; --k) { add_scaled(lin, b.var(k, nshape[k]), st); st *= nshape[k]; }
      st = 1;
      for (int k = rank - 1; k >= 0; --k) {            // split: old index k = (lin // stride_k) % extent_k
        Affine q = b.div(lin, st);
        subst[k] = (k == 0 && simplify) ? q : b.mod(q, shape[k]);
        st *= shape[k];
      }
      break;
    }
    default: *err = "unknown view operator"; return false;
  }
  std::vector<int> done(atoms.size(), 0);
  std::vector<Affine> memo(atoms.size());
  Affine noff = rebuild(atoms, offset, subst, b, done, memo);
  shape.swap(nshape);
  atoms.swap(fresh);
  offset = noff;
  return true;
}

int map_create(const std::vector<int64_t>& src_shape, const sm_view_op* chain, int n, sm_map** out, std::string* err) {
  if (src_shape.empty() || src_shape.size() > SM_MAX_RANK) { *err = "source rank out of range"; return SM_ERR_INVALID_ARG; }
  for (auto s : src_shape) if (s < 1) { *err = "source extent < 1"; return SM_ERR_SHAPE; }
  sm_map* m = new sm_map();
  m->src_shape = src_shape;
  m->shape = src_shape;
  {
    Builder b(m->atoms, true);
    int64_t st = 1;
    for (int k = (int)src_shape.size() - 1; k >= 0; --k) { add_scaled(m->offset, b.var(k, src_shape[k]), st); st *= src_shape[k]; }
  }
  // unsimplified twin, only to count what strength reduction removes
  std::vector<int64_t> rshape = src_shape; std::vector<Atom> ratoms = m->atoms; Affine roff = m->offset; int rmade = 0;
  int made = 0;
  for (int i = 0; i < n; ++i) {
    if (!apply_view(m->shape, m->atoms, m->offset, chain[i], true, &made, err)) { delete m; return SM_ERR_SHAPE; }
    std::string e2;
    apply_view(rshape, ratoms, roff, chain[i], false, &rmade, &e2);
    m->chain.push_back(chain[i]);
  }
  prune(m);
  {
    sm_map tmp; tmp.atoms = ratoms; tmp.offset = roff; prune(&tmp);
    m->n_divmod_raw = tmp.n_divmod();
  }
  *out = m;
  return SM_OK;
}

RowProg identity_rows(int64_t ld) {
  RowProg p; std::memset(&p, 0, sizeof(p));
  p.identity = 1; p.ld = ld;
  return p;
}

// Division by an invariant: for 0 <= x < 2^31 and d > 1, with l = ceil(log2 d) and m = ceil(2^(31+l) / d) < 2^32,
// floor(x / d) == (x * m) >> (31 + l) == umulhi(x, m) >> (l - 1).
void magic(int64_t d, uint32_t* mul, uint32_t* sh) {
  if (d <= 1) { *mul = 0; *sh = 0; return; }
  int l = 0;
  while ((int64_t(1) << l) < d) ++l;
  const unsigned __int128 num = (unsigned __int128)1 << (31 + l);
  *mul = (uint32_t)((num + d - 1) / d);
  *sh = (uint32_t)(l - 1);
}

template <class P>
static bool emit(const std::vector<Atom>& atoms, const Affine& offset, P* out, std::string* err) {
  // atoms are stored with arguments referring to earlier ids (intern order after prune)
  std::vector<int> slot(atoms.size(), 0), used(atoms.size(), 0);
  {
    std::vector<int> stack;
    for (auto& t : offset.terms) stack.push_back(t.first);
    while (!stack.empty()) {
      int id = stack.back(); stack.pop_back();
      if (used[id]) continue;
      used[id] = 1;
      for (auto& t : atoms[id].arg.terms) stack.push_back(t.first);
    }
  }
  int n = 0;
  for (size_t i = 0; i < atoms.size(); ++i) {
    const Atom& a = atoms[i];
    if (!used[i]) continue;
    if (a.kind == ATOM_VAR) { slot[i] = ~a.var; continue; }
    if (n >= PROG_MAX_ATOMS) { *err = "index map too complex for a device program (atoms)"; return false; }
    if ((int)a.arg.terms.size() > PROG_MAX_TERMS) { *err = "index map too complex for a device program (terms)"; return false; }
    ProgAtom& p = out->atoms[n];
    p.div = (int32_t)a.div; p.mod = (int32_t)a.mod; p.c0 = (int32_t)a.arg.c0; p.nterm = (int)a.arg.terms.size();
    magic(a.div, &p.div_mul, &p.div_sh);
    magic(a.mod, &p.mod_mul, &p.mod_sh);
    if (a.div > INT32_MAX || a.mod > INT32_MAX || a.arg.c0 > INT32_MAX || affine_hi(atoms, a.arg) > INT32_MAX) { *err = "index exceeds 32 bits"; return false; }
    for (int t = 0; t < p.nterm; ++t) {
      p.t_atom[t] = slot[a.arg.terms[t].first];
      p.t_coef[t] = (int32_t)a.arg.terms[t].second;
    }
    slot[i] = n++;
  }
  if ((int)offset.terms.size() > PROG_MAX_FINAL) { *err = "index map too complex for a device program (final)"; return false; }
  out->n_atoms = n; out->nterm = (int)offset.terms.size(); out->c0 = offset.c0;
  for (int t = 0; t < out->nterm; ++t) { out->t_atom[t] = slot[offset.terms[t].first]; out->t_coef[t] = offset.terms[t].second; }
  return true;
}

}  // namespace sm

using namespace sm;

int sm_map::n_divmod() const {
  int n = 0;
  for (auto& a : atoms) if (a.kind != ATOM_VAR) n += (a.div > 1) + (a.mod > 0);
  return n;
}

bool sm_map::compile(MapProg* out, std::string* err) const {
  std::memset(out, 0, sizeof(*out));
  out->rank = (int)shape.size();
  for (size_t k = 0; k < shape.size(); ++k) {
    if (shape[k] > INT32_MAX) { *err = "extent exceeds 32 bits"; return false; }
    out->shape[k] = (int32_t)shape[k];
  }
  return emit(atoms, offset, out, err);
}

bool sm_map::compile_rows(RowProg* out, std::string* err) const {
  std::memset(out, 0, sizeof(*out));
  const int64_t inner = shape.back();
  sm_map tmp = *this;
  sm_view_op rs; rs.kind = SM_VIEW_RESHAPE; rs.n = 2; rs.arg[0] = numel() / inner; rs.arg[1] = inner;
  int made = 0;
  if (!apply_view(tmp.shape, tmp.atoms, tmp.offset, rs, true, &made, err)) return false;
  prune(&tmp);
  // the inner variable must appear only as "+ 1 * i1" in the final expression
  int inner_atom = -1;
  for (size_t i = 0; i < tmp.atoms.size(); ++i)
    if (tmp.atoms[i].kind == ATOM_VAR && tmp.atoms[i].var == 1) inner_atom = (int)i;
  for (auto& a : tmp.atoms)
    for (auto& t : a.arg.terms)
      if (t.first == inner_atom) { *err = "operand's last dimension is not contiguous under the map"; return false; }
  Affine rows; rows.c0 = tmp.offset.c0;
  bool unit = inner == 1;
  for (auto& t : tmp.offset.terms) {
    if (t.first == inner_atom) { if (t.second != 1) { *err = "operand's last dimension has a stride"; return false; } unit = true; }
    else rows.terms.push_back(t);
  }
  if (!unit) { *err = "operand's last dimension is not addressed"; return false; }
  if (!emit(tmp.atoms, rows, out, err)) return false;
  // plain row-major rows?
  if (out->n_atoms == 0 && out->c0 == 0 && out->nterm == 1 && out->t_atom[0] == ~0) {
    out->identity = 1; out->ld = out->t_coef[0];
  }
  return true;
}

bool sm_map::compile_rows_cols(int gran, RowProg* rows, RowProg* cols, std::string* err) const {
  std::memset(rows, 0, sizeof(*rows)); std::memset(cols, 0, sizeof(*cols));
  const int64_t K = shape.back();
  if (K % gran) { *err = "last dimension is not a multiple of the granule"; return false; }
  sm_map tmp = *this;
  sm_view_op rs; rs.kind = SM_VIEW_RESHAPE; rs.n = 3; rs.arg[0] = numel() / K; rs.arg[1] = K / gran; rs.arg[2] = gran;
  int made = 0;
  if (!apply_view(tmp.shape, tmp.atoms, tmp.offset, rs, true, &made, err)) return false;
  prune(&tmp);
  // which view variables does each atom depend on (bit mask)
  std::vector<int> dep(tmp.atoms.size(), 0);
  for (size_t i = 0; i < tmp.atoms.size(); ++i) {
    const Atom& a = tmp.atoms[i];
    if (a.kind == ATOM_VAR) dep[i] = 1 << a.var;
    else for (auto& t : a.arg.terms) dep[i] |= dep[t.first];
  }
  Affine r_part, c_part;
  r_part.c0 = tmp.offset.c0;
  bool unit = gran == 1;
  for (auto& t : tmp.offset.terms) {
    const int d = dep[t.first];
    if (d == 1) r_part.terms.push_back(t);
    else if (d == 2) c_part.terms.push_back(t);
    else if (d == 4 && tmp.atoms[t.first].kind == ATOM_VAR && t.second == 1) unit = true;
    else { *err = "operand offset is not separable into row and column parts"; return false; }
  }
  if (!unit) { *err = "operand's innermost granule is not contiguous"; return false; }
  // column program: variable 1 becomes variable 0
  std::vector<Atom> catoms = tmp.atoms;
  for (auto& a : catoms) if (a.kind == ATOM_VAR && a.var == 1) a.var = 0; else if (a.kind == ATOM_VAR && a.var == 0) a.var = 1;
  if (!emit(tmp.atoms, r_part, rows, err)) return false;
  if (!emit(catoms, c_part, cols, err)) return false;
  return true;
}

void sm_map::eval(int64_t* offsets) const {
  const int rank = (int)shape.size();
  const int64_t n = numel();
  std::vector<int64_t> idx(rank, 0), val(atoms.size());
  for (int64_t o = 0; o < n; ++o) {
    for (size_t i = 0; i < atoms.size(); ++i) {
      const Atom& a = atoms[i];
      if (a.kind == ATOM_VAR) { val[i] = idx[a.var]; continue; }
      int64_t x = a.arg.c0;
      for (auto& t : a.arg.terms) x += t.second * val[t.first];
      x /= a.div;
      val[i] = a.mod ? x % a.mod : x;
    }
    int64_t off = offset.c0;
    for (auto& t : offset.terms) off += t.second * val[t.first];
    offsets[o] = off;
    for (int k = rank - 1; k >= 0; --k) { if (++idx[k] < shape[k]) break; idx[k] = 0; }
  }
}

int64_t sm_map::at(const int64_t* idx) const {
  std::vector<int64_t> val(atoms.size());
  for (size_t i = 0; i < atoms.size(); ++i) {
    const Atom& a = atoms[i];
    if (a.kind == ATOM_VAR) { val[i] = idx[a.var]; continue; }
    int64_t x = a.arg.c0;
    for (auto& t : a.arg.terms) x += t.second * val[t.first];
    x /= a.div;
    val[i] = a.mod ? x % a.mod : x;
  }
  int64_t off = offset.c0;
  for (auto& t : offset.terms) off += t.second * val[t.first];
  return off;
}

bool sm_map::inner_contiguous(int v) const {
  if (v == 1) return true;
  const int64_t last = shape.back();
  if (last % v) return false;
  sm_map tmp = *this;
  sm_view_op rs; rs.kind = SM_VIEW_RESHAPE; rs.n = (int)shape.size() + 1;
  if (rs.n > SM_MAX_RANK) return false;
  for (size_t k = 0; k + 1 < shape.size(); ++k) rs.arg[k] = shape[k];
  rs.arg[shape.size() - 1] = last / v; rs.arg[shape.size()] = v;
  int made = 0; std::string err;
  if (!apply_view(tmp.shape, tmp.atoms, tmp.offset, rs, true, &made, &err)) return false;
  prune(&tmp);
  const int inner = (int)tmp.shape.size() - 1;
  int inner_atom = -1;
  for (size_t i = 0; i < tmp.atoms.size(); ++i)
    if (tmp.atoms[i].kind == ATOM_VAR && tmp.atoms[i].var == inner) inner_atom = (int)i;
  if (inner_atom < 0) return false;
  for (auto& a : tmp.atoms)
    for (auto& t : a.arg.terms) if (t.first == inner_atom) return false;
  if (tmp.offset.c0 % v) return false;
  bool unit = false;
  for (auto& t : tmp.offset.terms) {
    if (t.first == inner_atom) unit = t.second == 1;
    else if (t.second % v) return false;
  }
  return unit;
}

bool sm_map::affine(int64_t* base, int64_t* strides) const {
  if (n_divmod() != 0) return false;
  for (size_t k = 0; k < SM_MAX_RANK; ++k) strides[k] = 0;
  *base = offset.c0;
  for (auto& t : offset.terms) strides[atoms[t.first].var] = t.second;
  return true;
}

namespace sm {
int64_t eval_rows_host(const RowProg& p, int64_t r) {
  if (p.identity) return r * p.ld;
  int64_t val[PROG_MAX_ATOMS] = {0};
  for (int i = 0; i < p.n_atoms; ++i) {
    const ProgAtom& a = p.atoms[i];
    int64_t x = a.c0;
    for (int t = 0; t < a.nterm; ++t) x += (int64_t)a.t_coef[t] * (a.t_atom[t] < 0 ? r : val[a.t_atom[t]]);
    if (a.div > 1) x /= a.div;
    if (a.mod >= 1) x %= a.mod;
    val[i] = x;
  }
  int64_t off = p.c0;
  for (int t = 0; t < p.nterm; ++t) off += p.t_coef[t] * (p.t_atom[t] < 0 ? r : val[p.t_atom[t]]);
  return off;
}
}  // namespace sm
