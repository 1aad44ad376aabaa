#include "expr.h"

#include <cmath>
#include <cstdio>
#include <cstring>
#include <map>
#include <tuple>

namespace fuse {

namespace {

bool is_unary(int op) { return op >= FUSE_OP_NEG && op <= FUSE_OP_SIGMOID; }
bool is_binary(int op) { return op >= FUSE_OP_ADD && op <= FUSE_OP_NE; }
bool zero_preserving_unary(int op)
{
    return op == FUSE_OP_NEG || op == FUSE_OP_ABS || op == FUSE_OP_SQRT || op == FUSE_OP_POW2 ||
           op == FUSE_OP_SIGN || op == FUSE_OP_NEQ0;
}

std::string lit(double v)
{
    char buf[64];
    if (std::isnan(v))
        return "__builtin_nan(\"\")";
    if (std::isinf(v))
        return v > 0 ? "__builtin_inf()" : "(-__builtin_inf())";
    std::snprintf(buf, sizeof buf, "%a", v);   // hex float: exact round trip
    return std::string("(") + buf + ")";
}

int fail(std::string &err, const std::string &msg)
{
    err = msg;
    return FUSE_EDESC;
}

}  // namespace

int parse_program(Tmpl t, const fuse_expr *exprs, int k, const fuse_side *sides, int nsides,
                  Program &prog, std::string &err, bool cell_body)
{
    const bool row = (t == Tmpl::ROW_DENSE || t == Tmpl::ROW_CSR);
    prog = Program();
    std::map<std::tuple<int, int, uint64_t, int, int>, int> seen;   // hash-consing of sub-expressions
    auto intern = [&](const Node &nd) {
        uint64_t bits;
        std::memcpy(&bits, &nd.imm, sizeof bits);
        const auto key = std::make_tuple(nd.op, nd.arg, bits, nd.a, nd.b);
        auto it = seen.find(key);
        if (it != seen.end())
            return it->second;
        prog.nodes.push_back(nd);
        seen[key] = (int)prog.nodes.size() - 1;
        return (int)prog.nodes.size() - 1;
    };
    for (int x = 0; x < k; ++x) {
        const fuse_expr &e = exprs[x];
        if (e.ntoks <= 0 || e.ntoks > 4096 || !e.toks) {
            err = "expression " + std::to_string(x) + ": empty, too long or NULL token list";
            return FUSE_EINVAL;
        }
        std::vector<int> st;
        for (int i = 0; i < e.ntoks; ++i) {
            const fuse_tok &tk = e.toks[i];
            const std::string at = "expression " + std::to_string(x) + ", token " + std::to_string(i) + ": ";
            Node nd;
            nd.op = tk.op;
            if (!st.empty() && prog.nodes[st.back()].kind == KIND_VK)
                return fail(err, at + "OUTERK must be the last token of a body");
            if (tk.op == FUSE_OP_MAIN) {
                nd.kind = row ? KIND_V : KIND_S;
                nd.zp = true;
            } else if (tk.op == FUSE_OP_SIDE) {
                if (tk.arg < 0 || tk.arg >= nsides)
                    return fail(err, at + "side index " + std::to_string(tk.arg) + " out of range");
                nd.arg = tk.arg;
                const int kind = sides[tk.arg].kind;
                if (kind == FUSE_SIDE_RHS || kind == FUSE_SIDE_KVEC) {
                    if (!row)
                        return fail(err, at + "right-hand-side and k-vector side inputs are only valid in a Row body");
                    const int kd = (int)sides[tk.arg].m.cols;
                    if (kd < 1 || kd > FUSE_MAX_K)
                        return fail(err, at + "k (columns of the side input) must be in [1, " +
                                             std::to_string(FUSE_MAX_K) + "]");
                    if (prog.kdim && prog.kdim != kd)
                        return fail(err, at + "all k-vectors of a body must have the same length");
                    prog.kdim = kd;
                    nd.kind = kind == FUSE_SIDE_RHS ? KIND_M : KIND_K;
                } else {
                    nd.kind = (row && (kind == FUSE_SIDE_MATRIX || kind == FUSE_SIDE_SPARSE || kind == FUSE_SIDE_ROWVEC)) ? KIND_V : KIND_S;
                }
                prog.side_used[tk.arg] = true;
            } else if (tk.op == FUSE_OP_CONST) {
                nd.imm = tk.imm;
            } else if (tk.op == FUSE_OP_UVDOT) {
                if (t != Tmpl::OUTER)
                    return fail(err, at + "UVDOT is only valid in an Outer body");
            } else if (is_unary(tk.op)) {
                if (st.empty())
                    return fail(err, at + "unary operator on an empty stack");
                nd.a = st.back();
                st.pop_back();
                const Node &a = prog.nodes[nd.a];
                if (a.kind == KIND_M)
                    return fail(err, at + "a right-hand side can only be consumed by MATMULT");
                nd.kind = a.kind;
                nd.level = a.level;
                nd.zp = a.kind == KIND_V && a.zp && zero_preserving_unary(tk.op);
            } else if (is_binary(tk.op)) {
                if (st.size() < 2)
                    return fail(err, at + "binary operator needs two operands");
                nd.b = st.back();
                st.pop_back();
                nd.a = st.back();
                st.pop_back();
                const Node &a = prog.nodes[nd.a], &b = prog.nodes[nd.b];
                if (a.kind == KIND_M || b.kind == KIND_M)
                    return fail(err, at + "a right-hand side can only be consumed by MATMULT");
                if ((a.kind == KIND_V && b.kind == KIND_K) || (a.kind == KIND_K && b.kind == KIND_V))
                    return fail(err, at + "a row vector and a k-vector do not conform");
                nd.kind = (a.kind == KIND_V || b.kind == KIND_V) ? KIND_V
                          : (a.kind == KIND_K || b.kind == KIND_K) ? KIND_K : KIND_S;
                nd.level = a.level > b.level ? a.level : b.level;
                if (nd.kind == KIND_V) {
                    const bool za = a.kind == KIND_V && a.zp, zb = b.kind == KIND_V && b.zp;
                    if (tk.op == FUSE_OP_MUL)
                        nd.zp = za || zb;
                    else if (tk.op == FUSE_OP_ADD || tk.op == FUSE_OP_SUB)
                        nd.zp = za && zb;
                    else if (tk.op == FUSE_OP_DIV)
                        nd.zp = za;
                    else
                        nd.zp = false;
                }
            } else if (tk.op == FUSE_OP_ROWSUM || tk.op == FUSE_OP_DOT) {
                if (!row)
                    return fail(err, at + "ROWSUM / DOT are only valid in a Row body");
                const size_t need = tk.op == FUSE_OP_DOT ? 2 : 1;
                if (st.size() < need)
                    return fail(err, at + "row aggregate needs more operands");
                if (tk.op == FUSE_OP_DOT) {
                    nd.b = st.back();
                    st.pop_back();
                }
                nd.a = st.back();
                st.pop_back();
                const Node &a = prog.nodes[nd.a];
                int lvl = a.level;
                if (nd.b >= 0 && prog.nodes[nd.b].level > lvl)
                    lvl = prog.nodes[nd.b].level;
                if (a.kind == KIND_K && (nd.b < 0 || prog.nodes[nd.b].kind == KIND_K)) {
                    // sum over the k entries of a per-row k-vector: plain scalar arithmetic
                    nd.kind = KIND_S;
                    nd.level = lvl;
                } else {
                    bool z = a.zp;
                    if (a.kind != KIND_V || (nd.b >= 0 && prog.nodes[nd.b].kind != KIND_V))
                        return fail(err, at + "row aggregate needs row vectors (or k-vectors)");
                    if (nd.b >= 0)
                        z = z || prog.nodes[nd.b].zp;
                    if (t == Tmpl::ROW_CSR && !z)
                        return fail(err, at + "not sparse-safe: row aggregate of a vector that is not zero "
                                              "where the main input has no stored cell");
                    nd.kind = KIND_S;
                    nd.level = lvl + 1;
                }
            } else if (tk.op == FUSE_OP_MATMULT) {
                if (!row)
                    return fail(err, at + "MATMULT is only valid in a Row body");
                if (st.size() < 2)
                    return fail(err, at + "MATMULT needs a row vector and a right-hand side");
                nd.b = st.back();
                st.pop_back();
                nd.a = st.back();
                st.pop_back();
                const Node &a = prog.nodes[nd.a], &b = prog.nodes[nd.b];
                if (a.kind != KIND_V || b.kind != KIND_M)
                    return fail(err, at + "MATMULT needs a row vector and a right-hand side");
                if (t == Tmpl::ROW_CSR && !a.zp)
                    return fail(err, at + "not sparse-safe: product of a vector that is not zero where the main "
                                          "input has no stored cell");
                nd.kind = KIND_K;
                nd.arg = b.arg;             // the right-hand side's side index
                nd.level = a.level + 1;
            } else if (tk.op == FUSE_OP_OUTERK) {
                if (!row)
                    return fail(err, at + "OUTERK is only valid in a Row body");
                if (st.size() < 2)
                    return fail(err, at + "OUTERK needs a row vector and a k-vector");
                nd.b = st.back();
                st.pop_back();
                nd.a = st.back();
                st.pop_back();
                const Node &a = prog.nodes[nd.a], &b = prog.nodes[nd.b];
                if (a.kind != KIND_V || b.kind != KIND_K)
                    return fail(err, at + "OUTERK needs a row vector and a k-vector");
                if (t == Tmpl::ROW_CSR && !a.zp)
                    return fail(err, at + "not sparse-safe: outer product of a vector that is not zero where the "
                                          "main input has no stored cell");
                nd.kind = KIND_VK;
                nd.level = a.level > b.level ? a.level : b.level;
            } else {
                return fail(err, at + "unknown opcode " + std::to_string(tk.op));
            }
            nd.vec = nd.kind == KIND_V;
            st.push_back(intern(nd));
        }
        if (st.size() != 1)
            return fail(err, "expression " + std::to_string(x) + " leaves " + std::to_string(st.size()) +
                                 " values on the stack");
        if (prog.nodes[st.back()].kind == KIND_M)
            return fail(err, "a right-hand side is not a result");
        prog.roots.push_back(st.back());
    }
    if (row) {
        const Node &r = prog.nodes[prog.roots[0]];
        const int rkind = (cell_body && r.kind == KIND_S) ? KIND_V : r.kind;
        prog.result_vec = rkind == KIND_V;
        prog.result_kind = rkind;
        for (int root : prog.roots) {
            const Node &q = prog.nodes[root];
            if (((cell_body && q.kind == KIND_S) ? KIND_V : q.kind) != rkind)
                return fail(err, "the results of a multi-aggregate must all be of the same kind");
            if (t == Tmpl::ROW_CSR && q.kind == KIND_V && !q.zp)
                return fail(err, "not sparse-safe: the result is not zero where the main input has no "
                                 "stored cell");
        }
        if (prog.roots.size() > 1 && rkind != KIND_V)
            return fail(err, "several results need row-vector bodies");
        // order the cross-lane reductions by stage (= level of the reduction node - 1)
        auto is_red = [&](const Node &n) {
            return n.op == FUSE_OP_MATMULT ||
                   ((n.op == FUSE_OP_ROWSUM || n.op == FUSE_OP_DOT) && prog.nodes[n.a].kind == KIND_V);
        };
        int maxlvl = 0;
        for (const Node &n : prog.nodes)
            if (is_red(n))
                maxlvl = n.level > maxlvl ? n.level : maxlvl;
        prog.nstage = maxlvl;
        for (int s = 0; s < maxlvl; ++s) {
            for (size_t i = 0; i < prog.nodes.size(); ++i) {
                Node &n = prog.nodes[i];
                if (is_red(n) && n.level == s + 1) {
                    n.red = prog.nred;
                    prog.nred += n.op == FUSE_OP_MATMULT ? prog.kdim : 1;
                    prog.reductions.push_back((int)i);
                }
            }
            prog.red_end.push_back(prog.nred);
        }
        if (prog.nred > 64)
            return fail(err, "more than 64 row-aggregate slots in one body");
    }
    return FUSE_OK;
}

std::string program_key(const Program &prog)
{
    std::string k;
    char buf[64];
    for (const Node &n : prog.nodes) {
        std::snprintf(buf, sizeof buf, "%d.%d.%a.%d.%d;", n.op, n.arg, n.op == FUSE_OP_CONST ? n.imm : 0.0, n.a, n.b);
        k += buf;
    }
    k += "|";
    for (int r : prog.roots)
        k += std::to_string(r) + ",";
    k += "|k" + std::to_string(prog.kdim) + "r" + std::to_string(prog.result_kind);    // widths the tokens do not show
    return k;
}

namespace {

// Emits the value of node `id` as C statements, one named constant per operator node (a body may
// be thousands of operators deep; nested as ONE expression it would exceed the compiler's bracket
// depth), and returns the operand text that stands for it.  `vec_side` / `scal_side`: names of the
// arrays that hold vector-kind and scalar-kind side values; cross-lane reductions that are already
// available are read from red[]; `d` is the Outer inner product.  For k-vector nodes `j` selects the
// component.  Statements collect in `stmts` (take() hands them over); names stay valid until reset().
struct Emitter {
    const Program &p;
    const char *vec_side;
    const char *scal_side;
    std::string indent = "    ";
    std::string stmts;
    std::map<std::pair<int, int>, std::string> done;

    void reset(const std::string &ind = "    ")
    {
        stmts.clear();
        done.clear();
        indent = ind;
    }
    std::string take()
    {
        std::string t;
        t.swap(stmts);
        return t;
    }
    std::string ref(int id, int j = 0)
    {
        const Node &n = p.nodes[id];
        switch (n.op) {
        case FUSE_OP_MAIN: return "a";
        case FUSE_OP_SIDE:
            if (n.kind == KIND_K)
                return "kv[" + std::to_string(n.arg * FUSE_MAX_K + j) + "]";
            return std::string(n.kind == KIND_V ? vec_side : scal_side) + "[" + std::to_string(n.arg) + "]";
        case FUSE_OP_CONST: return lit(n.imm);
        case FUSE_OP_UVDOT: return "d";
        case FUSE_OP_MATMULT: return "red[" + std::to_string(n.red + j) + "]";
        case FUSE_OP_ROWSUM:
        case FUSE_OP_DOT:
            if (n.red >= 0)
                return "red[" + std::to_string(n.red) + "]";
            break;
        default: break;
        }
        const int jj = n.kind == KIND_K ? j : 0;
        const auto key = std::make_pair(id, jj);
        auto it = done.find(key);
        if (it != done.end())
            return it->second;
        std::string e;
        if (n.op == FUSE_OP_ROWSUM || n.op == FUSE_OP_DOT) {      // over the k entries of k-vectors: written out
            for (int c = 0; c < p.kdim; ++c) {
                if (c)
                    e += " + ";
                e += n.op == FUSE_OP_DOT ? "(" + ref(n.a, c) + " * " + ref(n.b, c) + ")" : ref(n.a, c);
            }
        } else if (n.b < 0) {
            const std::string x = ref(n.a, j);
            switch (n.op) {
            case FUSE_OP_NEG: e = "-" + x; break;
            case FUSE_OP_ABS: e = "fabs(" + x + ")"; break;
            case FUSE_OP_SQRT: e = "sqrt(" + x + ")"; break;
            case FUSE_OP_EXP: e = "exp(" + x + ")"; break;
            case FUSE_OP_LOG: e = "log(" + x + ")"; break;
            case FUSE_OP_POW2: e = "fuse_pow2(" + x + ")"; break;
            case FUSE_OP_SIGN: e = "fuse_sign(" + x + ")"; break;
            case FUSE_OP_NEQ0: e = "fuse_neq0(" + x + ")"; break;
            case FUSE_OP_SIGMOID: e = "fuse_sigmoid(" + x + ")"; break;
            default: e = "0.0"; break;
            }
        } else {
            const std::string x = ref(n.a, j), y = ref(n.b, j);
            switch (n.op) {
            case FUSE_OP_ADD: e = x + " + " + y; break;
            case FUSE_OP_SUB: e = x + " - " + y; break;
            case FUSE_OP_MUL: e = x + " * " + y; break;
            case FUSE_OP_DIV: e = x + " / " + y; break;
            case FUSE_OP_MIN: e = "fuse_min(" + x + ", " + y + ")"; break;
            case FUSE_OP_MAX: e = "fuse_max(" + x + ", " + y + ")"; break;
            case FUSE_OP_POW: e = "pow(" + x + ", " + y + ")"; break;
            case FUSE_OP_LT: e = "fuse_cmp(" + x + " < " + y + ")"; break;
            case FUSE_OP_LE: e = "fuse_cmp(" + x + " <= " + y + ")"; break;
            case FUSE_OP_GT: e = "fuse_cmp(" + x + " > " + y + ")"; break;
            case FUSE_OP_GE: e = "fuse_cmp(" + x + " >= " + y + ")"; break;
            case FUSE_OP_EQ: e = "fuse_cmp(" + x + " == " + y + ")"; break;
            case FUSE_OP_NE: e = "fuse_cmp(" + x + " != " + y + ")"; break;
            default: e = "0.0"; break;
            }
        }
        const std::string name = "v" + std::to_string(id) + "_" + std::to_string(jj);
        stmts += indent + "const double " + name + " = " + e + ";\n";
        done[key] = name;
        return name;
    }
};

}  // namespace

std::string emit_cell_body(const Program &prog)
{
    Emitter em{prog, "s", "s"};
    std::string src = "__device__ __forceinline__ void fuse_body(double a, const double *s, double *r)\n{\n";
    for (size_t j = 0; j < prog.roots.size(); ++j) {
        const std::string v = em.ref(prog.roots[j]);
        src += em.take() + "    r[" + std::to_string(j) + "] = " + v + ";\n";
    }
    src += "}\n";
    return src;
}

std::string emit_outer_body(const Program &prog)
{
    Emitter em{prog, "s", "s"};
    const std::string v = em.ref(prog.roots[0]);
    return "__device__ __forceinline__ double fuse_body(double a, double d, const double *s)\n{\n" + em.take() +
           "    return " + v + ";\n}\n";
}

// Row bodies.  Arguments of the generated functions:
//   a    the main input's value at the current element of the row
//   sv   values of the vector-kind side inputs at that element        [FUSE_NSIDES]
//   kb   rows of the right-hand sides at that element's column        [FUSE_NSIDES * FUSE_MAX_K]
//   rsc  per-row scalars (column-vector and scalar sides)             [FUSE_NSIDES]
//   kv   per-row k-vectors (KVEC sides)                               [FUSE_NSIDES * FUSE_MAX_K]
//   red  finished cross-lane reductions of earlier stages             [FUSE_NRED]
std::string emit_row_body(const Program &prog)
{
    Emitter em{prog, "sv", "rsc"};
    const int kd = prog.kdim > 0 ? prog.kdim : 1;
    const int kres = prog.result_kind == KIND_VK || prog.result_kind == KIND_K ? kd : (int)prog.roots.size();
    std::string src;
    src += "#define FUSE_NSTAGE " + std::to_string(prog.nstage) + "\n";
    src += "#define FUSE_NRED " + std::to_string(prog.nred) + "\n";
    src += "#define FUSE_RESULT_VEC " + std::string(prog.result_vec ? "1" : "0") + "\n";
    src += "#define FUSE_RESULT_KIND " + std::to_string(prog.result_kind) + "\n";
    src += "#define FUSE_KDIM " + std::to_string(kd) + "\n";
    src += "#define FUSE_KRES " + std::to_string(kres) + "\n";
    src += "static __device__ constexpr int fuse_red_end[] = {";
    for (int e : prog.red_end)
        src += std::to_string(e) + ", ";
    src += "0};\n";
    // one partial-sum update per reduction slot, grouped by stage
    src += "__device__ __forceinline__ void fuse_stage(int st, double a, const double *sv, const double *kb,\n"
           "                                           const double *rsc, const double *kv, const double *red,\n"
           "                                           double *part)\n{\n";
    for (int s = 0; s < prog.nstage; ++s) {
        src += "    if (st == " + std::to_string(s) + ") {\n";
        em.reset("        ");
        for (int id : prog.reductions) {
            const Node &n = prog.nodes[id];
            if (n.level != s + 1)
                continue;
            if (n.op == FUSE_OP_MATMULT) {
                const std::string t = em.ref(n.a);
                src += em.take();
                for (int j = 0; j < prog.kdim; ++j)
                    src += "        part[" + std::to_string(n.red + j) + "] += " + t + " * kb[" +
                           std::to_string(n.arg * FUSE_MAX_K + j) + "];\n";
            } else {
                const std::string x = em.ref(n.a);
                const std::string term = n.op == FUSE_OP_DOT ? x + " * " + em.ref(n.b) : x;
                src += em.take() + "        part[" + std::to_string(n.red) + "] += " + term + ";\n";
            }
        }
        src += "    }\n";
    }
    src += "}\n";
    const int root = prog.roots[0];
    // row-vector results (k of them for a multi-aggregate), or row (x) k-vector: k values per element
    src += "__device__ __forceinline__ void fuse_final_elems(double a, const double *sv, const double *rsc,\n"
           "                                                 const double *kv, const double *red, double *r)\n{\n";
    em.reset();
    if (prog.result_kind == KIND_VK) {
        const Node &n = prog.nodes[root];
        const std::string t = em.ref(n.a);
        src += em.take();
        for (int j = 0; j < kd; ++j) {
            const std::string w = em.ref(n.b, j);
            src += em.take() + "    r[" + std::to_string(j) + "] = " + t + " * " + w + ";\n";
        }
    } else {
        for (int j = 0; j < kres; ++j) {
            const std::string v = prog.result_kind == KIND_V ? em.ref(prog.roots[j]) : std::string("0.0");
            src += em.take() + "    r[" + std::to_string(j) + "] = " + v + ";\n";
        }
    }
    src += "}\n";
    // the k-vector factor of a row (x) k-vector result on its own (the matrix-unit skeleton forms the
    // outer products itself)
    src += "__device__ __forceinline__ void fuse_outer_kvec(const double *rsc, const double *kv, const double *red,\n"
           "                                                double *r)\n{\n";
    em.reset();
    for (int j = 0; j < kd; ++j) {
        const std::string v = prog.result_kind == KIND_VK ? em.ref(prog.nodes[root].b, j) : std::string("0.0");
        src += em.take() + "    r[" + std::to_string(j) + "] = " + v + ";\n";
    }
    src += "}\n";
    src += "__device__ __forceinline__ double fuse_final_elem(double a, const double *sv, const double *rsc,\n"
           "                                                  const double *kv, const double *red)\n{\n";
    em.reset();
    {
        const std::string v = prog.result_kind == KIND_V ? em.ref(root) : std::string("0.0");
        src += em.take() + "    return " + v + ";\n}\n";
    }
    src += "__device__ __forceinline__ double fuse_final_scalar(const double *rsc, const double *kv,\n"
           "                                                    const double *red)\n{\n";
    em.reset();
    {
        const std::string v = prog.result_kind == KIND_S ? em.ref(root) : std::string("0.0");
        src += em.take() + "    return " + v + ";\n}\n";
    }
    src += "__device__ __forceinline__ void fuse_final_kvec(const double *rsc, const double *kv, const double *red,\n"
           "                                                double *r)\n{\n";
    em.reset();
    for (int j = 0; j < kd; ++j) {
        const std::string v = prog.result_kind == KIND_K ? em.ref(root, j) : std::string("0.0");
        src += em.take() + "    r[" + std::to_string(j) + "] = " + v + ";\n";
    }
    src += "}\n";
    return src;
}

}  // namespace fuse
