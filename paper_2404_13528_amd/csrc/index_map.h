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
  const int32_t* table;    // device memory or null: the program evaluated for rows 0 .. n-1 (attach_row_table)
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
// Evaluates the program for rows 0 .. n_rows-1 on the host and leaves the offsets in device memory that lives
// until the process ends (plans are cached for that long); kernels then read one word per row instead of
// interpreting the program.  No table (and success) for identity programs and for offsets beyond 31 bits.
bool attach_row_table(RowProg* p, int64_t n_rows, std::string* err);
}
