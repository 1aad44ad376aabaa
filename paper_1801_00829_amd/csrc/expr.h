// Expression descriptor -> typed tree -> HIP source of the generated body.
// Host-side analogue of CPlan construction and template expansion
// (Sec. 2.2 "Code Generation Plans": a template node holding a DAG of basic
// operations, expanded depth-first into source).
#pragma once
#include <cstdint>
#include <string>
#include <vector>

#include "../../include/fuse.h"

namespace fuse {

enum class Tmpl { CELL, ROW_DENSE, ROW_CSR, OUTER };

// Kinds of values in a body.  Cell / Outer bodies only have scalars (per cell /
// per non-zero).  Row bodies: per-row scalar, row vector (n), per-row k-vector
// (result of a product with an n x k right-hand side, or a KVEC side), the
// right-hand side itself, and row (x) k-vector (n x k per row; result only).
enum Kind { KIND_S = 0, KIND_V = 1, KIND_K = 2, KIND_M = 3, KIND_VK = 4 };

struct Node {
    int op = 0;
    int arg = 0;
    double imm = 0.0;
    int a = -1, b = -1;      // operand node ids
    int kind = KIND_S;
    bool vec = false;        // kind == KIND_V
    int level = 0;           // number of cross-lane reductions below this node
    bool zp = false;         // row vector is zero wherever the main input has no stored cell
    int red = -1;            // first reduction slot (ROWSUM / DOT over columns: 1 slot; MATMULT: k slots)
};

struct Program {
    std::vector<Node> nodes;
    std::vector<int> roots;          // one per expression (MAgg: k)
    std::vector<int> reductions;     // node ids of cross-lane reductions, ordered by stage
    std::vector<int> red_end;        // red_end[s] = number of reduction SLOTS in stages <= s
    int nred = 0;                    // total number of reduction slots
    int nstage = 0;
    bool result_vec = false;         // Row: the result is a row vector
    int result_kind = KIND_S;        // Row: kind of the (first) root
    int kdim = 0;                    // length of k-vectors (0: none in this body)
    bool side_used[8] = {false, false, false, false, false, false, false, false};
    std::string key;                 // canonical text (program_key), filled by parse_cached
};

// Parse and type-check `k` postfix expressions for a template.  side kinds
// decide the kind of a SIDE token in a Row body.  Equal sub-expressions become
// one node (a row aggregate that occurs twice is computed once).  Returns
// FUSE_OK or FUSE_EDESC / FUSE_EINVAL / FUSE_EUNSUPPORTED with a message in err.
// cell_body (Row templates): the expressions are Cell bodies evaluated per cell of the row, so a
// result without any row-vector operand (only scalars / column-vector sides) still counts as a row
// vector: it is the same value at every cell of the row.
int parse_program(Tmpl t, const fuse_expr *exprs, int k, const fuse_side *sides, int nsides,
                  Program &prog, std::string &err, bool cell_body = false);

// Canonical text of a program (cache key part).
std::string program_key(const Program &prog);

// Body source for the Cell / MAgg skeleton: fuse_body(a, s, r).
std::string emit_cell_body(const Program &prog);
// Body source for the Outer skeleton: fuse_body(a, d, s) -> double.
std::string emit_outer_body(const Program &prog);
// Body source for the Row skeletons: stage functions, final element / scalar /
// k-vector functions, FUSE_NSTAGE, FUSE_NRED, fuse_red_end[], FUSE_RESULT_KIND,
// FUSE_KRES, FUSE_KMAX.
std::string emit_row_body(const Program &prog);

}  // namespace fuse
