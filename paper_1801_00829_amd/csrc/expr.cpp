#include "expr.h"

#include <cmath>
#include <cstdio>
#include <cstring>

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
                  Program &prog, std::string &err)
{
    const bool row = (t == Tmpl::ROW_DENSE || t == Tmpl::ROW_CSR);
    prog = Program();
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
            if (tk.op == FUSE_OP_MAIN) {
                nd.vec = row;
                nd.zp = true;
            } else if (tk.op == FUSE_OP_SIDE) {
                if (tk.arg < 0 || tk.arg >= nsides)
                    return fail(err, at + "side index " + std::to_string(tk.arg) + " out of range");
                nd.arg = tk.arg;
                const int kind = sides[tk.arg].kind;
                nd.vec = row && (kind == FUSE_SIDE_MATRIX || kind == FUSE_SIDE_ROWVEC);
                nd.zp = false;
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
                nd.vec = a.vec;
                nd.level = a.level;
                nd.zp = a.vec && a.zp && zero_preserving_unary(tk.op);
            } else if (is_binary(tk.op)) {
                if (st.size() < 2)
                    return fail(err, at + "binary operator needs two operands");
                nd.b = st.back();
                st.pop_back();
                nd.a = st.back();
                st.pop_back();
                const Node &a = prog.nodes[nd.a], &b = prog.nodes[nd.b];
                nd.vec = a.vec || b.vec;
                nd.level = a.level > b.level ? a.level : b.level;
                if (nd.vec) {
                    const bool za = a.vec && a.zp, zb = b.vec && b.zp;
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
                bool z = a.zp;
                int lvl = a.level;
                if (!a.vec || (nd.b >= 0 && !prog.nodes[nd.b].vec))
                    return fail(err, at + "row aggregate of a scalar");
                if (nd.b >= 0) {
                    z = z || prog.nodes[nd.b].zp;
                    if (prog.nodes[nd.b].level > lvl)
                        lvl = prog.nodes[nd.b].level;
                }
                if (t == Tmpl::ROW_CSR && !z)
                    return fail(err, at + "not sparse-safe: row aggregate of a vector that is not zero "
                                          "where the main input has no stored cell");
                nd.vec = false;
                nd.level = lvl + 1;
            } else {
                return fail(err, at + "unknown opcode " + std::to_string(tk.op));
            }
            prog.nodes.push_back(nd);
            st.push_back((int)prog.nodes.size() - 1);
        }
        if (st.size() != 1)
            return fail(err, "expression " + std::to_string(x) + " leaves " + std::to_string(st.size()) +
                                 " values on the stack");
        prog.roots.push_back(st.back());
    }
    if (row) {
        const Node &r = prog.nodes[prog.roots[0]];
        prog.result_vec = r.vec;
        for (int root : prog.roots) {
            const Node &q = prog.nodes[root];
            if (q.vec != r.vec)
                return fail(err, "the results of a multi-aggregate must all be of the same kind");
            if (t == Tmpl::ROW_CSR && q.vec && !q.zp)
                return fail(err, "not sparse-safe: the result is not zero where the main input has no "
                                 "stored cell");
        }
        // order reductions by stage (= level of the reduction node - 1)
        int maxlvl = 0;
        for (const Node &n : prog.nodes)
            if (n.op == FUSE_OP_ROWSUM || n.op == FUSE_OP_DOT)
                maxlvl = n.level > maxlvl ? n.level : maxlvl;
        prog.nstage = maxlvl;
        for (int s = 0; s < maxlvl; ++s) {
            for (size_t i = 0; i < prog.nodes.size(); ++i) {
                Node &n = prog.nodes[i];
                if ((n.op == FUSE_OP_ROWSUM || n.op == FUSE_OP_DOT) && n.level == s + 1) {
                    n.red = (int)prog.reductions.size();
                    prog.reductions.push_back((int)i);
                }
            }
            prog.red_end.push_back((int)prog.reductions.size());
        }
        if (prog.reductions.size() > 32)
            return fail(err, "more than 32 row aggregates in one body");
    }
    return FUSE_OK;
}

std::string program_key(const Program &prog)
{
    std::string k;
    char buf[64];
    for (const Node &n : prog.nodes) {
        std::snprintf(buf, sizeof buf, "%d.%d.%a;", n.op, n.arg, n.op == FUSE_OP_CONST ? n.imm : 0.0);
        k += buf;
    }
    k += "|";
    for (int r : prog.roots)
        k += std::to_string(r) + ",";
    return k;
}

namespace {

// Emits node `id` as a C expression.  `vec_side`/`scal_side`: names of the
// arrays that hold vector-kind and scalar-kind side values; reductions that are
// already available are read from red[]; `d` is the Outer inner product.
struct Emitter {
    const Program &p;
    const char *vec_side;
    const char *scal_side;
    std::string gen(int id) const
    {
        const Node &n = p.nodes[id];
        switch (n.op) {
        case FUSE_OP_MAIN: return "a";
        case FUSE_OP_SIDE: return std::string(n.vec ? vec_side : scal_side) + "[" + std::to_string(n.arg) + "]";
        case FUSE_OP_CONST: return lit(n.imm);
        case FUSE_OP_UVDOT: return "d";
        case FUSE_OP_ROWSUM:
        case FUSE_OP_DOT: return "red[" + std::to_string(n.red) + "]";
        default: break;
        }
        if (n.b < 0) {
            const std::string x = gen(n.a);
            switch (n.op) {
            case FUSE_OP_NEG: return "(-" + x + ")";
            case FUSE_OP_ABS: return "fabs(" + x + ")";
            case FUSE_OP_SQRT: return "sqrt(" + x + ")";
            case FUSE_OP_EXP: return "exp(" + x + ")";
            case FUSE_OP_LOG: return "log(" + x + ")";
            case FUSE_OP_POW2: return "fuse_pow2(" + x + ")";
            case FUSE_OP_SIGN: return "fuse_sign(" + x + ")";
            case FUSE_OP_NEQ0: return "fuse_neq0(" + x + ")";
            case FUSE_OP_SIGMOID: return "fuse_sigmoid(" + x + ")";
            }
        }
        const std::string x = gen(n.a), y = gen(n.b);
        switch (n.op) {
        case FUSE_OP_ADD: return "(" + x + " + " + y + ")";
        case FUSE_OP_SUB: return "(" + x + " - " + y + ")";
        case FUSE_OP_MUL: return "(" + x + " * " + y + ")";
        case FUSE_OP_DIV: return "(" + x + " / " + y + ")";
        case FUSE_OP_MIN: return "fuse_min(" + x + ", " + y + ")";
        case FUSE_OP_MAX: return "fuse_max(" + x + ", " + y + ")";
        case FUSE_OP_POW: return "pow(" + x + ", " + y + ")";
        case FUSE_OP_LT: return "fuse_cmp(" + x + " < " + y + ")";
        case FUSE_OP_LE: return "fuse_cmp(" + x + " <= " + y + ")";
        case FUSE_OP_GT: return "fuse_cmp(" + x + " > " + y + ")";
        case FUSE_OP_GE: return "fuse_cmp(" + x + " >= " + y + ")";
        case FUSE_OP_EQ: return "fuse_cmp(" + x + " == " + y + ")";
        case FUSE_OP_NE: return "fuse_cmp(" + x + " != " + y + ")";
        }
        return "0.0";
    }
};

}  // namespace

std::string emit_cell_body(const Program &prog)
{
    Emitter em{prog, "s", "s"};
    std::string src = "__device__ __forceinline__ void fuse_body(double a, const double *s, double *r)\n{\n";
    for (size_t j = 0; j < prog.roots.size(); ++j)
        src += "    r[" + std::to_string(j) + "] = " + em.gen(prog.roots[j]) + ";\n";
    src += "}\n";
    return src;
}

std::string emit_outer_body(const Program &prog)
{
    Emitter em{prog, "s", "s"};
    return "__device__ __forceinline__ double fuse_body(double a, double d, const double *s)\n{\n"
           "    return " + em.gen(prog.roots[0]) + ";\n}\n";
}

std::string emit_row_body(const Program &prog)
{
    Emitter em{prog, "sv", "rsc"};
    std::string src;
    src += "#define FUSE_NSTAGE " + std::to_string(prog.nstage) + "\n";
    src += "#define FUSE_NRED " + std::to_string(prog.reductions.size()) + "\n";
    src += "#define FUSE_RESULT_VEC " + std::string(prog.result_vec ? "1" : "0") + "\n";
    src += "static __device__ constexpr int fuse_red_end[] = {";
    for (int e : prog.red_end)
        src += std::to_string(e) + ", ";
    src += "0};\n";
    // one partial-sum update per reduction, grouped by stage
    src += "__device__ __forceinline__ void fuse_stage(int st, double a, const double *sv, const double *rsc,\n"
           "                                           const double *red, double *part)\n{\n";
    int begin = 0;
    for (int s = 0; s < prog.nstage; ++s) {
        src += "    if (st == " + std::to_string(s) + ") {\n";
        for (int i = begin; i < prog.red_end[s]; ++i) {
            const Node &n = prog.nodes[prog.reductions[i]];
            std::string term = n.op == FUSE_OP_DOT ? "(" + em.gen(n.a) + " * " + em.gen(n.b) + ")" : em.gen(n.a);
            src += "        part[" + std::to_string(i) + "] += " + term + ";\n";
        }
        src += "    }\n";
        begin = prog.red_end[s];
    }
    src += "}\n";
    const int root = prog.roots[0];
    src += "#define FUSE_KRES " + std::to_string(prog.roots.size()) + "\n";
    src += "__device__ __forceinline__ void fuse_final_elems(double a, const double *sv, const double *rsc,\n"
           "                                                 const double *red, double *r)\n{\n";
    for (size_t j = 0; j < prog.roots.size(); ++j)
        src += "    r[" + std::to_string(j) + "] = " +
               (prog.result_vec ? em.gen(prog.roots[j]) : std::string("0.0")) + ";\n";
    src += "}\n";
    src += "__device__ __forceinline__ double fuse_final_elem(double a, const double *sv, const double *rsc,\n"
           "                                                  const double *red)\n{\n    return " +
           (prog.result_vec ? em.gen(root) : std::string("0.0")) + ";\n}\n";
    src += "__device__ __forceinline__ double fuse_final_scalar(const double *rsc, const double *red)\n{\n"
           "    return " + (prog.result_vec ? std::string("0.0") : em.gen(root)) + ";\n}\n";
    return src;
}

}  // namespace fuse
