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

struct Node {
    int op = 0;
    int arg = 0;
    double imm = 0.0;
    int a = -1, b = -1;      // operand node ids
    bool vec = false;        // Row: row vector (true) or per-row scalar (false)
    int level = 0;           // number of reductions below this node
    bool zp = false;         // vector is zero wherever the main input has no stored cell
    int red = -1;            // reduction number (ROWSUM / DOT nodes)
};

struct Program {
    std::vector<Node> nodes;
    std::vector<int> roots;          // one per expression (MAgg: k)
    std::vector<int> reductions;     // node ids ordered by stage
    std::vector<int> red_end;        // red_end[s] = number of reductions in stages <= s
    int nstage = 0;
    bool result_vec = false;         // Row: kind of the (single) root
    bool side_used[8] = {false, false, false, false, false, false, false, false};
};

// Parse and type-check `k` postfix expressions for a template.  side kinds
// decide whether a SIDE token is a vector or a scalar in a Row body.  Returns
// FUSE_OK or FUSE_EDESC / FUSE_EINVAL with a message in err.
int parse_program(Tmpl t, const fuse_expr *exprs, int k, const fuse_side *sides, int nsides,
                  Program &prog, std::string &err);

// Canonical text of a program (cache key part).
std::string program_key(const Program &prog);

// Body source for the Cell / MAgg skeleton: fuse_body(a, s, r).
std::string emit_cell_body(const Program &prog);
// Body source for the Outer skeleton: fuse_body(a, d, s) -> double.
std::string emit_outer_body(const Program &prog);
// Body source for the Row skeletons: stage functions, final element / scalar,
// FUSE_NSTAGE, FUSE_NRED, fuse_red_end[], FUSE_RESULT_VEC.
std::string emit_row_body(const Program &prog);

}  // namespace fuse
