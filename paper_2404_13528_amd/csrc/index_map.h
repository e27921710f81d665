// Index-map composer: symbolic index expressions over view variables, built
// from identity / split (//, %) / merge (*, +) dependencies and simplified with
// exact strength-reduction rules (paper Sec. 3.2.1).
#pragma once
#include <cstdint>
#include <string>
#include <vector>
#include "../../include/smartmem.h"

namespace sm {

// affine combination of atoms with non-negative integer coefficients
struct Affine {
  int64_t c0 = 0;
  std::vector<std::pair<int, int64_t>> terms;   // (atom id, coefficient), sorted by atom id
};

// An atom is a view variable or a "digit" (arg // div) % mod of an affine
// argument; mod == 0 means no modulus, div == 1 no division.
enum AtomKind { ATOM_VAR = 0, ATOM_DIGIT = 1 };
struct Atom {
  int kind;
  int var;          // ATOM_VAR: view axis
  Affine arg;       // ATOM_DIGIT argument
  int64_t div, mod;
  int64_t hi;       // inclusive upper bound of the atom's value (lower bound is 0)
};

// Fixed-size compiled form handed to device kernels by value.
constexpr int PROG_MAX_ATOMS = 16;
constexpr int PROG_MAX_TERMS = 6;
constexpr int PROG_MAX_FINAL = 12;
struct ProgAtom {
  int32_t div; int32_t mod; int32_t c0; int32_t nterm;   // value = (c0 + sum coef*term) / div % mod (mod 0: none)
  uint32_t div_mul, div_sh, mod_mul, mod_sh;             // x / d == umulhi(x, mul) >> sh for 0 <= x < 2^31 (d > 1)
  int32_t t_atom[PROG_MAX_TERMS];      // >= 0: earlier atom; < 0: view variable ~t_atom
  int32_t t_coef[PROG_MAX_TERMS];
};
struct MapProg {
  int32_t rank; int32_t n_atoms; int32_t nterm; int32_t pad;
  int64_t c0;
  int32_t shape[SM_MAX_RANK];
  int32_t t_atom[PROG_MAX_FINAL];
  int64_t t_coef[PROG_MAX_FINAL];
  ProgAtom atoms[PROG_MAX_ATOMS];
};

// Row program: offset of row r of a [rows, inner] view whose inner dimension is
// contiguous; one variable.
struct RowProg {
  int32_t identity;        // 1: offset = r * ld
  int32_t n_atoms; int32_t nterm; int32_t pad;
  int64_t ld;              // identity only
  int64_t c0;
  const int32_t* table;    // device memory or null: the program evaluated for rows 0 .. n-1; kernels read one word per
                           // row instead of interpreting the program
  int64_t table_off;       // host bookkeeping: byte offset + 1 of that table inside its plan's table region, 0 = no table
  int32_t t_atom[PROG_MAX_FINAL];
  int64_t t_coef[PROG_MAX_FINAL];
  ProgAtom atoms[PROG_MAX_ATOMS];
};

}  // namespace sm

struct sm_map {
  std::vector<int64_t> src_shape;
  std::vector<int64_t> shape;            // current view shape
  std::vector<sm::Atom> atoms;           // interned; arguments refer to earlier atoms only
  sm::Affine offset;                     // source element offset
  int n_divmod_raw = 0;                  // // and % count without simplification
  std::vector<sm_view_op> chain;         // as given (for compose)

  int64_t numel() const { int64_t n = 1; for (auto s : shape) n *= s; return n; }
  int n_divmod() const;
  bool compile(sm::MapProg* out, std::string* err) const;
  // view collapsed to [rows, inner]: inner = last axis, must be contiguous
  bool compile_rows(sm::RowProg* out, std::string* err) const;
  // view collapsed to [rows, K / gran, gran] with offset = rows_part(r) + cols_part(k / gran) + k % gran
  bool compile_rows_cols(int gran, sm::RowProg* rows, sm::RowProg* cols, std::string* err) const;
  void eval(int64_t* offsets) const;
  int64_t at(const int64_t* idx) const;       // offset of one view element
  bool affine(int64_t* base, int64_t* strides) const;
  // true if every aligned group of v consecutive elements of the last view axis is contiguous in the source
  // and starts at an offset that is a multiple of v
  bool inner_contiguous(int v) const;
};

namespace sm {
int map_create(const std::vector<int64_t>& src_shape, const sm_view_op* chain, int n, sm_map** out, std::string* err);
RowProg identity_rows(int64_t ld);
// x / d == umulhi(x, *mul) >> *sh for 0 <= x < 2^31 and d > 1 (d <= 1: both zero, callers test d)
void magic(int64_t d, uint32_t* mul, uint32_t* sh);
int64_t eval_rows_host(const RowProg& p, int64_t r);
// Per-row offset tables.  A plan (host memory only) lists the row programs that want a table and gives each a slot
// in a "table region"; the executor places the region in the caller's workspace, fills it on the caller's stream
// with one small kernel per table (fill_tables) at the start of every call, and hands kernels copies of the
// programs whose `table` points into it (bound).  Nothing is allocated and nothing outlives the call.
struct TableRegion {
  struct Item { RowProg prog; int64_t n_rows; size_t off; };
  std::vector<Item> items;
  size_t bytes = 0;
  // gives p a slot when every offset fits 31 bits (src_numel = elements of the tensor the offsets point into);
  // identity programs need none
  void add(RowProg* p, int64_t n_rows, int64_t src_numel);
};
// which: bit i set = fill the i-th added program's table (tables no kernel of the call reads can be left out)
int fill_tables(const TableRegion& r, void* region, void* stream, uint64_t which);     // SM_OK or SM_ERR_DEVICE
inline RowProg bound(const RowProg& p, const void* region) {
  RowProg q = p;
  q.table = (p.table_off && region) ? (const int32_t*)((const char*)region + (p.table_off - 1)) : nullptr;
  return q;
}
}
