// libfuse C ABI: validation, kernel selection and launch for the four template
// entry points (see include/fuse.h for the contract of every call).
#include "../../include/fuse.h"

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <memory>
#include <mutex>
#include <new>
#include <stdexcept>
#include <string>
#include <unordered_map>

#include "expr.h"
#include "runtime.h"

namespace {

using namespace fuse;

// ---- skeleton sources, embedded as text --------------------------------------
const char *kSrcArgs =
#include "gen_args_text.inc"
    ;
const char *kSrcCommon =
#include "skel_common.inc"
    ;
const char *kSrcCell =
#include "skel_cell.inc"
    ;
const char *kSrcRowDense =
#include "skel_row_dense.inc"
    ;
const char *kSrcRowMfma =
#include "skel_row_mfma.inc"
    ;
const char *kSrcRowMfmaWave =
#include "skel_row_mfma_wave.inc"
    ;
const char *kSrcRowCsr =
#include "skel_row_csr.inc"
    ;
const char *kSrcRowCsrStream =
#include "skel_row_csr_stream.inc"
    ;
const char *kSrcOuter =
#include "skel_outer.inc"
    ;

// Parsed descriptors by their raw bytes (template, tokens, side kinds): a call with a descriptor
// seen before skips parsing, typing and the canonical key text -- the steady state of an operator
// that is called in a loop (Sec. 2.1: "plan cache" lookups must be cheap next to a small operator).
struct ParsedEntry {
    int rc = 0;
    std::string err;
    Program prog;
};
std::mutex g_parse_mu;
std::unordered_map<std::string, std::shared_ptr<const ParsedEntry>> g_parsed;

int parse_cached(Tmpl t, const fuse_expr *exprs, int k, const fuse_side *sides, int nsides, Program &prog,
                 std::string &err, bool cell_body = false)
{
    std::string raw;
    raw.reserve(256);
    auto put = [&](const void *p, size_t n) { raw.append(static_cast<const char *>(p), n); };
    const int head[4] = {(int)t, (int)cell_body, k, nsides};
    put(head, sizeof head);
    bool ok = exprs != nullptr && k >= 1 && k <= FUSE_MAX_AGGS && nsides >= 0 && nsides <= FUSE_MAX_SIDES &&
              (nsides == 0 || sides != nullptr);
    for (int x = 0; ok && x < k; ++x) {
        if (!exprs[x].toks || exprs[x].ntoks < 0 || exprs[x].ntoks > 4096) {
            ok = false;
            break;
        }
        put(&exprs[x].ntoks, sizeof exprs[x].ntoks);
        for (int q = 0; q < exprs[x].ntoks; ++q) {
            const fuse_tok &tk = exprs[x].toks[q];
            put(&tk.op, sizeof tk.op);
            put(&tk.arg, sizeof tk.arg);
            put(&tk.imm, sizeof tk.imm);
        }
    }
    if (!ok)                                   // malformed: let the parser produce the message
        return parse_program(t, exprs, k, sides, nsides, prog, err, cell_body);
    for (int q = 0; q < nsides; ++q) {
        const long long kc[2] = {sides[q].kind, (sides[q].kind == FUSE_SIDE_RHS || sides[q].kind == FUSE_SIDE_KVEC)
                                                    ? (long long)sides[q].m.cols : 0};
        put(kc, sizeof kc);
    }
    {
        std::lock_guard<std::mutex> lk(g_parse_mu);
        auto it = g_parsed.find(raw);
        if (it != g_parsed.end()) {
            prog = it->second->prog;
            err = it->second->err;
            return it->second->rc;
        }
    }
    auto e = std::make_shared<ParsedEntry>();
    e->rc = parse_program(t, exprs, k, sides, nsides, e->prog, e->err, cell_body);
    if (e->rc == 0)
        e->prog.key = program_key(e->prog);
    prog = e->prog;
    err = e->err;
    std::lock_guard<std::mutex> lk(g_parse_mu);
    if (g_parsed.size() > 4096)
        g_parsed.clear();
    g_parsed.emplace(std::move(raw), e);
    return e->rc;
}

thread_local std::string g_err;
thread_local std::string g_last_source;
thread_local std::string g_last_kernel;

int fail(int code, const std::string &msg)
{
    g_err = msg;
    return code;
}

int env_int(const char *name, int dflt)
{
    const char *e = std::getenv(name);
    return (e && *e) ? std::atoi(e) : dflt;
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int next_pow2(int64_t v)
{
    int p = 1;
    while (p < v)
        p <<= 1;
    return p;
}

struct SideInfo {
    int kind[FUSE_MAX_SIDES];
};

// Shape checks shared by all templates: side k against an m x n main input.
int check_sides(const fuse_side *sides, int nsides, int64_t m, int64_t n, bool need_data,
                const bool *used, bool sparse_ok = false)
{
    if (nsides < 0 || nsides > FUSE_MAX_SIDES)
        return fail(FUSE_EINVAL, "nsides must be in [0, " + std::to_string(FUSE_MAX_SIDES) + "]");
    if (nsides > 0 && !sides)
        return fail(FUSE_EINVAL, "sides is NULL");
    for (int k = 0; k < nsides; ++k) {
        const fuse_side &s = sides[k];
        const std::string at = "side " + std::to_string(k) + ": ";
        switch (s.kind) {
        case FUSE_SIDE_MATRIX:
            if (s.m.rows != m || s.m.cols != n)
                return fail(FUSE_ESHAPE, at + "matrix side must be " + std::to_string(m) + " x " + std::to_string(n));
            if (s.m.ld < n)
                return fail(FUSE_ESHAPE, at + "ld < cols");
            break;
        case FUSE_SIDE_COLVEC:
            if (s.m.rows != m || s.m.cols != 1)
                return fail(FUSE_ESHAPE, at + "column-vector side must be " + std::to_string(m) + " x 1");
            if (s.m.ld < 1)
                return fail(FUSE_ESHAPE, at + "ld < 1");
            break;
        case FUSE_SIDE_ROWVEC:
            if (s.m.rows != 1 || s.m.cols != n)
                return fail(FUSE_ESHAPE, at + "row-vector side must be 1 x " + std::to_string(n));
            break;
        case FUSE_SIDE_SCALAR:
            break;
        case FUSE_SIDE_RHS:
            if (s.m.rows != n || s.m.cols < 1 || s.m.cols > FUSE_MAX_K)
                return fail(FUSE_ESHAPE, at + "right-hand side must be " + std::to_string(n) + " x k, 1 <= k <= " +
                                             std::to_string(FUSE_MAX_K));
            if (s.m.ld < s.m.cols)
                return fail(FUSE_ESHAPE, at + "ld < cols");
            break;
        case FUSE_SIDE_KVEC:
            if (s.m.rows != m || s.m.cols < 1 || s.m.cols > FUSE_MAX_K)
                return fail(FUSE_ESHAPE, at + "k-vector side must be " + std::to_string(m) + " x k, 1 <= k <= " +
                                             std::to_string(FUSE_MAX_K));
            if (s.m.ld < s.m.cols)
                return fail(FUSE_ESHAPE, at + "ld < cols");
            break;
        case FUSE_SIDE_SPARSE: {
            if (!sparse_ok)
                return fail(FUSE_EUNSUPPORTED, at + "sparse side inputs go with a CSR main input (fuse_cell_csr, fuse_magg_csr, fuse_row with Xs)");
            const fuse_csr *c = s.sp;
            if (!c)
                return fail(FUSE_EINVAL, at + "sp is NULL");
            if (c->rows != m || c->cols != n)
                return fail(FUSE_ESHAPE, at + "sparse side must be " + std::to_string(m) + " x " + std::to_string(n));
            if (c->nnz < 0 || (!c->rowptr_is64 && c->nnz > 2147483647LL))
                return fail(FUSE_EINVAL, at + "bad nnz for the offset width");
            if (need_data && used[k] && (!c->rowptr || (c->nnz > 0 && (!c->vals || !c->colidx))) && m > 0)
                return fail(FUSE_EINVAL, at + "array pointer of the sparse side is NULL");
            continue;
        }
        default:
            return fail(FUSE_EINVAL, at + "unknown side kind " + std::to_string(s.kind));
        }
        if (need_data && used[k] && s.kind != FUSE_SIDE_SCALAR && !s.m.data && m * n > 0)
            return fail(FUSE_EINVAL, at + "data is NULL");
    }
    return 0;
}

int check_dense(const fuse_dense *X, const char *what, bool need_data)
{
    if (!X)
        return fail(FUSE_EINVAL, std::string(what) + " is NULL");
    if (X->rows < 0 || X->cols < 0)
        return fail(FUSE_EINVAL, std::string(what) + ": negative shape");
    if (X->ld < X->cols)
        return fail(FUSE_ESHAPE, std::string(what) + ": ld < cols");
    if (need_data && !X->data && X->rows * X->cols > 0)
        return fail(FUSE_EINVAL, std::string(what) + ": data is NULL");
    return 0;
}

int check_csr(const fuse_csr *X, bool need_data)
{
    if (!X)
        return fail(FUSE_EINVAL, "X is NULL");
    if (X->rows < 0 || X->cols < 0 || X->nnz < 0)
        return fail(FUSE_EINVAL, "X: negative shape or nnz");
    if (X->cols > 2147483647LL)
        return fail(FUSE_EUNSUPPORTED, "X: more than 2^31-1 columns (int32 column indices)");
    if (!X->rowptr_is64 && X->nnz > 2147483647LL)
        return fail(FUSE_EINVAL, "X: nnz does not fit the int32 row offsets");
    if (X->cols == 0 || X->rows <= (int64_t)4e18 / X->cols) {       // rows * cols representable
        if (X->nnz > X->rows * X->cols)
            return fail(FUSE_ESHAPE, "X: nnz exceeds rows * cols");
    }
    if (need_data && (!X->rowptr || (X->nnz > 0 && (!X->vals || !X->colidx))))
        return fail(FUSE_EINVAL, "X: NULL CSR array");
    return 0;
}

std::string side_tables(const fuse_side *sides, int nsides, const bool *used)
{
    std::string s = "#define FUSE_NSIDES " + std::to_string(nsides) + "\n";
    s += "static __device__ constexpr int fuse_side_kind[] = {";
    for (int k = 0; k < nsides; ++k)
        s += std::to_string(sides[k].kind) + ", ";
    s += "-1};\nstatic __device__ constexpr bool fuse_side_used[] = {";
    for (int k = 0; k < nsides; ++k)
        s += std::string(used[k] ? "true" : "false") + ", ";
    s += "false};\nstatic __device__ constexpr bool fuse_side_rp64[] = {";      // sparse sides: 64-bit row offsets
    for (int k = 0; k < nsides; ++k)
        s += std::string(sides[k].kind == FUSE_SIDE_SPARSE && sides[k].sp && sides[k].sp->rowptr_is64 ? "true" : "false") + ", ";
    s += "false};\n";
    return s;
}

std::string side_key(const fuse_side *sides, int nsides)
{
    std::string s = "sides:";
    for (int k = 0; k < nsides; ++k) {
        s += std::to_string(sides[k].kind);
        if (sides[k].kind == FUSE_SIDE_SPARSE)
            s += (sides[k].sp && sides[k].sp->rowptr_is64) ? "L" : "l";
    }
    return s;
}

void fill_side_args(fuse_kargs &A, const fuse_side *sides, int nsides)
{
    for (int k = 0; k < nsides; ++k) {
        if (sides[k].kind == FUSE_SIDE_SPARSE && sides[k].sp) {
            A.side[k] = sides[k].sp->vals;
            A.side_ci[k] = sides[k].sp->colidx;
            A.side_rp[k] = sides[k].sp->rowptr;
            A.side_ld[k] = sides[k].sp->nnz;                  // bound of every offset read from side_rp
            continue;
        }
        A.side[k] = sides[k].m.data;
        A.side_ld[k] = sides[k].kind == FUSE_SIDE_ROWVEC ? 0 : sides[k].m.ld;
        A.side_scalar[k] = sides[k].scalar;
    }
}

int zero_fill(Plan::Loaded &fn, double *out, int64_t count, hipStream_t stream)
{
    if (count <= 0)
        return 0;
    struct {
        double *out;
        long long n;
        double v;
    } a = {out, count, 0.0};
    unsigned gx = (unsigned)std::min<int64_t>((count + 255) / 256, 1024);
    return Runtime::get().launch(fn.fill, gx, 1, 256, stream, &a, sizeof a, g_err);
}

int run_combine(Plan::Loaded &fn, const double *partials, int nblocks, int nv, double *out,
                hipStream_t stream)
{
    struct {
        const double *partials;
        int nblocks, nv;
        double *out;
    } a = {partials, nblocks, nv, out};
    return Runtime::get().launch(fn.combine, (unsigned)((nv + 3) / 4), 1, 256, stream, &a, sizeof a, g_err);
}

int agg_code(int agg)
{
    switch (agg) {
    case FUSE_AGG_NONE: return 0;
    case FUSE_AGG_FULL: return 1;
    case FUSE_AGG_ROW: return 2;
    case FUSE_AGG_COL:
    case FUSE_AGG_COL_T: return 3;
    }
    return -1;
}

// ------------------------------------------------------------ row (dense, MFMA) --
// Bodies  t(X) %*% W  with  W_i = f(X_i %*% V, per-row sides):  exactly one MATMULT of the main
// input with a right-hand side, and an OUTERK of the main input with a k-vector as the result.
bool mfma_pattern(const Program &prog, const fuse_side *sides, int nsides, int &vside)
{
    if (prog.result_kind != KIND_VK || prog.nstage != 1 || prog.reductions.size() != 1 || prog.roots.size() != 1)
        return false;
    const Node &mm = prog.nodes[prog.reductions[0]];
    const Node &root = prog.nodes[prog.roots[0]];
    if (mm.op != FUSE_OP_MATMULT || root.op != FUSE_OP_OUTERK)
        return false;
    if (prog.nodes[mm.a].op != FUSE_OP_MAIN || prog.nodes[root.a].op != FUSE_OP_MAIN)
        return false;
    const Node &v = prog.nodes[mm.b];
    if (v.op != FUSE_OP_SIDE || v.arg < 0 || v.arg >= nsides || sides[v.arg].kind != FUSE_SIDE_RHS)
        return false;
    for (int q = 0; q < nsides; ++q)
        if (prog.side_used[q] && (sides[q].kind == FUSE_SIDE_MATRIX || sides[q].kind == FUSE_SIDE_SPARSE || sides[q].kind == FUSE_SIDE_ROWVEC))
            return false;
    vside = v.arg;
    return true;
}

// one wave per 16-row tile: at most 7 column tiles, contiguous rows
bool mfma_wave_form(const fuse_dense *X, bool launch)
{
    return X->cols <= 112 && X->ld == X->cols && (!launch || aligned16(X->data)) && env_int("FUSE_MFMA_WAVE_FORM", 1) != 0;
}

// X: the dense main input, or nullptr with Xs the CSR main input (block form only: its rows are spread out
// into the dense LDS tile).
int row_mfma_impl(const Program &prog, const std::string &pkey, const fuse_dense *X, const fuse_csr *Xs, const fuse_side *sides,
                  int nsides, int vside, double *out, hipStream_t stream, bool launch)
{
    Runtime &rt = Runtime::get();
    const int64_t m = X ? X->rows : Xs->rows, n = X ? X->cols : Xs->cols;
    const int kd = prog.kdim;
    const bool vec2 = X && (n % 2 == 0) && (X->ld % 2 == 0) && (!launch || aligned16(X->data));
    const int VEC = vec2 ? 2 : 1;
    const int64_t nct = (n + 15) / 16;                       // 16-column tiles
    const int64_t np = nct * 16 + 1;                         // odd LDS row pitch
    const int64_t nvec = (n + VEC - 1) / VEC;
    // few columns and contiguous rows: every wave works alone on its own tiles (FUSE_MFMA_WAVE_FORM=0: never).
    // Measured on 3.2 GB, t(X)(XV) / logistic regression core, k = 8, against the block form below: n = 16
    // 1.3 / 1.7 against 3.7 / 5.4 ms, n = 32 0.94 / 1.36 against 2.1 / 2.9, n = 64 0.83 / 1.13 against 1.26 / 1.56,
    // n = 100 0.86 / 1.10 against 1.15 / 1.23; with 8 column tiles (n = 128) the registers no longer hold the
    // travelling tile, V and the running sums (0.93 / 1.18 - 1.45 against 0.95 / 1.0 - 1.1): the block form stays.
    if (X && mfma_wave_form(X, launch)) {
        const int64_t lds = (16 * np + 16 * 17) * 8;
        // Bodies with per-row k-vector sides hold k-vectors next to V, the running sums and the travelling tile:
        // for them the next tile starts travelling only after the generated code has run (its registers are free
        // for the body), and from 13 classes on the registers are budgeted for one wave per SIMD (512) instead of
        // two (256 each).  1e7 x 100, multinomial logistic regression core, early / late fetch: k = 8 2.42 / 1.67 ms
        // (one wave per SIMD: 2.22 / 2.15), k = 12 3.77 / 2.19 (2.32 / 2.19), k = 16 5.90 / 3.16 (2.45 / 2.29); with the
        // 4x4x4 products (k <= 8), on 3.2 GB: k = 8 1318 / 793 us, k = 5 777 / 753, k = 4 508 / 523, k = 2 491 / 523.
        bool kvec_side = false;
        for (int q = 0; q < nsides; ++q)
            kvec_side = kvec_side || (prog.side_used[q] && sides[q].kind == FUSE_SIDE_KVEC);
        int wpe = env_int("FUSE_MFMA_WPE", 0);
        // Narrow tiles (n <= 32: 2 - 4 KB) leave a wave waiting on its own chain of LDS and MFMA latencies, and need
        // few registers: four waves per SIMD there (3.2 GB, t(X)(XV): n = 16, k = 4 1129 -> 766 us, n = 32 758 -> 530;
        // at n = 32 with k-vector sides of 16 classes it spilled: 2.6 against 1.1 ms)
        if (wpe != 1 && wpe != 2 && wpe != 4 && wpe != 8)
            wpe = (kvec_side && kd > 12) ? 1 : (n <= 32 && !(kvec_side && kd > 8)) ? 4 : 2;
        // Bodies with per-row k-vector sides of more than 12 classes: 4x4x4 products with V in LDS, shared by the four
        // waves of a block, which frees V's registers for the body at two waves per SIMD (FUSE_MFMA_VLDS: 0 never,
        // 1 whenever k > 8).  6.4 GB, logistic regression core, k = 16, against 16x16x4 with V in registers and one
        // wave per SIMD: n = 100 1562 against 2083 us, n = 64 2176 against 2199, n = 32 2505 against 2694.  Elsewhere
        // the B operand read from LDS per product costs more than the higher instruction rate gains (t(X)(XV),
        // k = 9 / 12 / 16: n = 100 1591 / 1650 / 1533 against 1554 / 1580 / 1646 us, n = 64 1584 / 1626 / 1930
        // against 1559 / 1619 / 1642, n = 32 1791 / 1849 / 2076 against 1551 / 1607 / 1698).
        const int vlds_env = env_int("FUSE_MFMA_VLDS", -1);
        const int vlds = vlds_env == 0 ? 0 : vlds_env == 1 ? (kd > 8) : (kvec_side && kd > 12);
        if (vlds && env_int("FUSE_MFMA_WPE", 0) == 0)
            wpe = 2;
        int late = env_int("FUSE_MFMA_FETCH_LATE", -1);
        if (late != 0 && late != 1)
            late = (kvec_side && kd > 4) ? 1 : 0;
        const std::string key = std::string("rowmfmaw|") + pkey + "|" + side_key(sides, nsides) + "|n" + std::to_string(n) +
                                "nt" + std::to_string(env_int("FUSE_NT", 1)) + "e" + std::to_string(wpe) + "l" + std::to_string(late) + "v" + std::to_string(vlds);
        std::shared_ptr<Plan> plan;
        int rc = rt.plan(key, "fuse_row_mfma_wave", [&](const std::string &name) {
            std::string s = kSrcArgs;
            s += "#define FUSE_NT " + std::to_string(env_int("FUSE_NT", 1)) + "\n";
            s += kSrcCommon;
            s += "#define FUSE_KERNEL_NAME " + name + "\n";
            s += "#define FUSE_NCOLS " + std::to_string(n) + "\n#define FUSE_NP " + std::to_string(np) + "\n#define FUSE_NCT " +
                 std::to_string(nct) + "\n#define FUSE_VSIDE " + std::to_string(vside) + "\n#define FUSE_WPE " + std::to_string(wpe) + "\n#define FUSE_FETCH_LATE " + std::to_string(late) + "\n#define FUSE_VLDS " + std::to_string(vlds) + "\n";
            s += side_tables(sides, nsides, prog.side_used);
            s += emit_row_body(prog);
            s += kSrcRowMfmaWave;
            g_last_source = s;
            return s;
        }, plan, g_err);
        if (rc)
            return rc;
        g_last_kernel = plan->kernel_name;
        if (!launch)
            return 0;
        Plan::Loaded fn;
        if ((rc = rt.load(*plan, fn, g_err)))
            return rc;
        if (m == 0 || n == 0)
            return zero_fill(fn, out, n * kd, stream);
        const int64_t ntiles = (m + 15) / 16;
        // one-wave blocks: as many per CU as their LDS tiles allow, at most 8 (two per SIMD: their registers)
        const int bw = vlds ? 4 : 1;          // waves per block
        const int64_t lds_block = bw * lds + (vlds ? (n + 3) / 4 * 4 * 16 * 8 : 0);
        const int64_t wpc = std::max<int64_t>(bw, std::min<int64_t>((160 * 1024) / lds_block * bw, env_int("FUSE_MFMA_WAVES_PER_CU", 4 * wpe)));
        const int64_t gx = std::max<int64_t>(1, std::min<int64_t>((ntiles + bw - 1) / bw, (int64_t)rt.num_cus() * wpc / bw));
        Workspace ws;
        if ((rc = rt.workspace(stream, (size_t)gx * bw * (size_t)(n * kd), ws, g_err)))
            return rc;
        fuse_kargs A;
        std::memset(&A, 0, sizeof A);
        A.x = X->data;
        A.m = m;
        A.n = n;
        A.ld = X->ld;
        A.out = out;
        A.partials = ws.partials;
        A.ticket = ws.ticket;
        fill_side_args(A, sides, nsides);
        if ((rc = rt.launch(fn.main, (unsigned)gx, 1, 64 * bw, stream, &A, sizeof A, g_err)))
            return rc;
        // (a wave of the last block without a tile still writes its partial sums: zeros)
        return run_combine(fn, ws.partials, (int)(gx * bw), (int)(n * kd), out, stream);
    }
    // waves per block (FUSE_MFMA_WAVES, default 8), fewer if the LDS next to the tile does not hold that many
    // partial products (16 x 17 doubles each)
    int NWAVE = env_int("FUSE_MFMA_WAVES", 8);
    if (NWAVE != 4 && NWAVE != 8 && NWAVE != 16)
        NWAVE = 8;
    const int ns_ = std::max(nsides, 1);
    auto lds_bytes = [&](int nw) { return (16 * np + (int64_t)(nw + 2 + ns_) * 272 + (int64_t)ns_ * 16) * 8; };
    while (NWAVE > 4 && lds_bytes(NWAVE) > 158 * 1024)
        NWAVE >>= 1;
    if (lds_bytes(NWAVE) > 158 * 1024)
        return fail(FUSE_EUNSUPPORTED, "internal: matrix-unit Row form chosen for a row tile that does not fit in LDS");
    const int BLOCK = 64 * NWAVE;
    const int64_t nld = (nvec + BLOCK / 16 - 1) / (BLOCK / 16);
    // 4x4x4 products up to 4 classes (less padding, a higher instruction rate; FUSE_MFMA_M4: 0 never, 1 always).
    // With more groups of 4 classes V's operands take one register pair per group and column step of the wave:
    // 1e6 x 784, k = 10 spilled (4.6 against 1.6 ms); 1e6 x 256, k = 8: 365 / 588 against 443 / 469 us
    // (t(X)(XV) / logistic regression core); k = 4: 1e6 x 784 1.17 / 1.19 against 1.61 / 1.66 ms, 3e6 x 128
    // 0.67 / 0.72 against 0.91 / 0.97 ms.
    int m4 = env_int("FUSE_MFMA_M4", -1);
    if (m4 != 0 && m4 != 1)
        m4 = kd <= 4 ? 1 : 0;
    // CSR input: cells per thread that travel in registers (the mean row length and a third, over the threads of a row)
    const int csrx = Xs != nullptr;
    const int rp64 = Xs && Xs->rowptr_is64;
    int cap = 1;
    if (Xs) {
        const double avg = m > 0 ? (double)Xs->nnz / (double)m : 1.0;
        cap = (int)std::min<int64_t>(16, std::max<int64_t>(1, (int64_t)(avg * 1.34 / (BLOCK / 16)) + 1));
    }
    const std::string key = std::string("rowmfma|") + pkey + "|" + side_key(sides, nsides) + "|v" + std::to_string(VEC) +
                            "n" + std::to_string(nct) + "w" + std::to_string(NWAVE) + "nt" + std::to_string(env_int("FUSE_NT", 1)) +
                            "m" + std::to_string(m4) + (csrx ? "csr" + std::to_string(rp64) + "c" + std::to_string(cap) : "");
    std::shared_ptr<Plan> plan;
    int rc = rt.plan(key, "fuse_row_mfma", [&](const std::string &name) {
        std::string s = kSrcArgs;
        s += "#define FUSE_NT " + std::to_string(env_int("FUSE_NT", 1)) + "\n";
        s += kSrcCommon;
        s += "#define FUSE_KERNEL_NAME " + name + "\n";
        s += "#define FUSE_M4 " + std::to_string(m4) + "\n";
        s += "#define FUSE_CSRX " + std::to_string(csrx) + "\n#define FUSE_RP64 " + std::to_string(rp64) + "\n#define FUSE_CAP " +
             std::to_string(cap) + "\n";
        s += "#define FUSE_NWAVE " + std::to_string(NWAVE) + "\n#define FUSE_VEC " + std::to_string(VEC) + "\n#define FUSE_NP " + std::to_string(np) +
             "\n#define FUSE_NCT " + std::to_string(nct) + "\n#define FUSE_NLD " + std::to_string(nld) +
             "\n#define FUSE_VSIDE " + std::to_string(vside) + "\n";
        s += side_tables(sides, nsides, prog.side_used);
        s += emit_row_body(prog);
        s += kSrcRowMfma;
        g_last_source = s;
        return s;
    }, plan, g_err);
    if (rc)
        return rc;
    g_last_kernel = plan->kernel_name;
    if (!launch)
        return 0;
    Plan::Loaded fn;
    if ((rc = rt.load(*plan, fn, g_err)))
        return rc;
    if (m == 0 || n == 0)
        return zero_fill(fn, out, n * kd, stream);
    const int64_t ntiles = (m + 15) / 16;
    // as many blocks per CU as their tiles fit in LDS (and the register file: 512 / waves-per-SIMD): the phases
    // of one block (tile store, Q, body, H) then overlap with another block's
    const int64_t by_lds = std::max<int64_t>(1, (158 * 1024) / lds_bytes(NWAVE));
    const int64_t bpc = std::max<int64_t>(1, std::min<int64_t>(std::min<int64_t>(by_lds, 16 / NWAVE),
                                                            env_int("FUSE_MFMA_BLOCKS_PER_CU", 4)));
    const int64_t gx = std::max<int64_t>(1, std::min<int64_t>(ntiles, (int64_t)rt.num_cus() * bpc));
    Workspace ws;
    if ((rc = rt.workspace(stream, (size_t)gx * (size_t)(n * kd), ws, g_err)))
        return rc;
    fuse_kargs A;
    std::memset(&A, 0, sizeof A);
    if (X) {
        A.x = X->data;
        A.ld = X->ld;
    } else {
        A.x = Xs->vals;
        A.colidx = Xs->colidx;
        A.rowptr = Xs->rowptr;
        A.nnz = Xs->nnz;
        A.ld = n;
    }
    A.m = m;
    A.n = n;
    A.out = out;
    A.partials = ws.partials;
    A.ticket = ws.ticket;
    fill_side_args(A, sides, nsides);
    if ((rc = rt.launch(fn.main, (unsigned)gx, 1, BLOCK, stream, &A, sizeof A, g_err)))
        return rc;
    return run_combine(fn, ws.partials, (int)gx, (int)(n * kd), out, stream);
}

// ------------------------------------------------------------------ row (dense) --
// Shared by fuse_row (dense) and by Cell bodies that need the 2-D form.
int row_dense_impl(const Program &prog, const std::string &pkey, const fuse_dense *X,
                   const fuse_side *sides, int nsides, int agg, double *out, hipStream_t stream,
                   bool launch, const char *name_prefix)
{
    Runtime &rt = Runtime::get();
    const int64_t m = X->rows, n = X->cols;
    const int ac = agg_code(agg);
    const int rk = prog.result_kind;
    if (rk == KIND_S && (ac == 2 || ac == 3))
        return fail(FUSE_EDESC, "row / column aggregation needs a row-vector result");
    if (rk == KIND_K && ac == 2)
        return fail(FUSE_EDESC, "a k-vector result has the variants no_agg, col_agg and full_agg");
    if (rk == KIND_VK && ac != 3)
        return fail(FUSE_EDESC, "an OUTERK result needs FUSE_AGG_COL / FUSE_AGG_COL_T");
    const int kd = prog.kdim;

    // matrix-unit form: from FUSE_MFMA_MIN_K classes on, while 16 rows of X fit in LDS (about 1200 columns)
    {
        int vside = -1;
        // (measured against the vector form: equal at k = 4 for n = 784, 2.6x faster at k = 8 for n = 256,
        //  3.2x at k = 10 for n = 784; slower for k = 4 at n = 100 and n = 1000)
        //  (that was with 16x16x4 products; with 4x4x4 products k = 4 wins at every width measured, on 3.2 GB,
        //  t(X)(XV) / logistic regression core: n = 128 744 / 798 against 801 / 987 us, n = 256 584 / 613 against
        //  871 / 992, n = 500 713 / 738 against 736 / 822, n = 784 626 / 665 against 1107 / 1149, n = 1000 639 / 676
        //  against 886 / 879; k = 3 wins at n = 256 and 784 but loses at 128, 500 and 1000);
        //  with one wave per tile (few columns, contiguous rows; 4x4x4 products up to 8 classes) the matrix units
        //  win earlier, the wider the rows are -- 3.2 GB, t(X)(XV) / logistic regression core, vector against
        //  matrix units: n = 100 k = 2 510 / 530 against 486 / 500 us (k = 1: 463 / 469 against 480 / 493);
        //  n = 64 k = 3 645 / 761 against 561 / 562 (k = 2: 487 / 509 against 638 / 546); n = 32 k = 3 646 / 828
        //  against 537 / 562 (k = 2: 500 / 502 against 521 / 524); n = 24 k = 3 780 / 979 against 699 / 625;
        //  n = 16 k = 5 1029 / 1573 against 896 / 941 (k = 4: 724 / 995 against 793 / 896); after 25 calls, when
        //  both forms have sped up: n = 16 k = 4 625 / 774 against 611 / 683 (k = 3: 534 / 670 against 600 / 665),
        //  n = 64 k = 2 479 / 517 against 474 / 490, n = 32 k = 2 480 / 513 against 500 / 531, n = 100 k = 1
        //  462 / 470 against 481 / 490; block form: n = 256 k = 3 615 / 661 against 516 / 511 and n = 784 k = 3
        //  742 / 736 against 597 / 622, but n = 128 k = 3 570 / 644 against 659 / 734, n = 500 k = 4 630 / 672
        //  against 676 / 723, n = 1000 k = 3 516 / 547 against 594 / 609: the rule for the block form stays at 4)
        int min_k = env_int("FUSE_MFMA_MIN_K", -1);
        if (min_k < 0)
            min_k = !mfma_wave_form(X, launch) ? 4 : n >= 48 ? 2 : n > 16 ? 3 : 4;
        const int64_t tile_bytes = (16 * ((n + 15) / 16 * 16 + 1) + (int64_t)(4 + 2 + std::max(nsides, 1)) * 272 + 128) * 8;
        if (ac == 3 && min_k > 0 && kd >= min_k && n >= 16 && tile_bytes <= 158 * 1024 &&
            mfma_pattern(prog, sides, nsides, vside))
            return row_mfma_impl(prog, pkey, X, nullptr, sides, nsides, vside, out, stream, launch);
    }

    // vector width: 16-byte loads need even strides and aligned bases
    bool vec2 = (n % 2 == 0) && (X->ld % 2 == 0) && (!launch || aligned16(X->data));
    for (int k = 0; k < nsides && vec2; ++k) {
        if (!prog.side_used[k])
            continue;
        if (sides[k].kind == FUSE_SIDE_MATRIX)
            vec2 = (sides[k].m.ld % 2 == 0) && (!launch || aligned16(sides[k].m.data));
        else if (sides[k].kind == FUSE_SIDE_ROWVEC)
            vec2 = !launch || aligned16(sides[k].m.data);
    }
    if (ac == 0 && prog.result_vec && launch && !aligned16(out))
        vec2 = false;
    const int VEC = vec2 ? 2 : 1;
    const int64_t nvec = (n + VEC - 1) / VEC;
    // lanes per row and vectors per lane
    int epl_target = env_int("FUSE_ROW_EPL", 4);
    if (kd > 0)      // k values per owned column are kept in registers (right-hand side, accumulators)
        epl_target = std::max(1, std::min(epl_target, 16 / (VEC * kd)));
    int G = 1;
    while (G < 64 && (nvec + G - 1) / G > epl_target)
        G <<= 1;
    int64_t epl64 = (nvec + G - 1) / G;
    int stripes = 1;
    int WPR = 1;                 // waves per row (> 1: the whole block owns one row)
    // registers a lane spends per owned column: the row itself, and with k-vectors the k entries of the
    // right-hand side and of the accumulators
    auto fits = [&](int64_t epl) { return epl <= 16 && (kd == 0 || epl * VEC * kd <= 48); };
    if (!fits(epl64)) {
        if (prog.nstage > 0 || kd > 0) {
            // per-row reductions over a row wider than one wave's registers: 2 .. 16 waves per row
            G = 64;
            epl64 = (nvec + 63) / 64;
            while (WPR < 16 && !fits(epl64)) {
                WPR <<= 1;
                epl64 = (nvec + (int64_t)64 * WPR - 1) / ((int64_t)64 * WPR);
            }
            if (!fits(epl64))
                return fail(FUSE_EUNSUPPORTED,
                            kd > 0 ? "Row bodies with k-vectors need ceil(cols / " + std::to_string(1024 * VEC) + ") * " +
                                         std::to_string(VEC) + " * k <= 48 in this build"
                                   : "Row bodies with ROWSUM / DOT need cols <= " + std::to_string(64 * 16 * 16 * VEC) +
                                         " for dense input");
        } else {
            epl64 = 16;
            stripes = (int)((n + (int64_t)64 * 16 * VEC - 1) / ((int64_t)64 * 16 * VEC));
        }
    }
    if (epl64 < 1)
        epl64 = 1;
    const int EPL = (int)epl64;
    int RS = env_int("FUSE_ROW_RS", 0);
    if (RS <= 0)
        RS = EPL >= 8 ? 1 : (EPL >= 3 ? 2 : 4);
    const int BLOCK = WPR > 1 ? std::max(128, 64 * WPR) : 256;
    if (WPR > 1 && BLOCK != 64 * WPR)
        WPR = BLOCK / 64;          // at least two waves per block
    if (WPR > 1)          // (more rows in flight per block were tried: no gain at k = 4, spills at k = 10)
        RS = 1;

    // contiguous rows that are narrow (at most 8 lanes per row; with 8-byte vectors, an odd row length, at
    // most 32: beyond that the direct loads of a row are long enough and 5.8 against 6.7 TB/s were measured
    // at 301 columns): the wave's rows are fetched as one contiguous span with 16-byte loads and handed out through LDS
    // (FUSE_ROW_LDSX=0 switches it off); the span is a whole number of 16-byte vectors, at most 8 KB
    bool ldsx = WPR == 1 && stripes == 1 && (G <= 8 || (VEC == 1 && G <= 32)) && n >= 1 && X->ld == n && (!launch || aligned16(X->data)) &&
                env_int("FUSE_ROW_LDSX", 1) != 0;
    if (ldsx && VEC == 1 && env_int("FUSE_ROW_RS", 0) <= 0)
        RS = EPL <= 4 ? 4 : (EPL <= 8 ? 2 : 1);        // 8-byte vectors: more rows per pass, the same registers
    {
        const int64_t span = (int64_t)(64 / G) * RS * n;
        if (span % 2 != 0 || span > 1024)
            ldsx = false;
    }
    const std::string key = std::string("rowdense|") + pkey + "|rk" + std::to_string(rk) + "|" + side_key(sides, nsides) + "|agg" +
                            std::to_string(ac) + "|v" + std::to_string(VEC) + "g" + std::to_string(G) + "e" +
                            std::to_string(EPL) + "r" + std::to_string(RS) + "w" + std::to_string(WPR) + "nt" +
                            std::to_string(env_int("FUSE_NT", 1)) + (ldsx ? "x" + std::to_string(n) : "");
    std::shared_ptr<Plan> plan;
    int rc = rt.plan(key, name_prefix, [&](const std::string &name) {
        std::string s = kSrcArgs;
        s += "#define FUSE_NT " + std::to_string(env_int("FUSE_NT", 1)) + "\n";
        s += kSrcCommon;
        s += "#define FUSE_KERNEL_NAME " + name + "\n";
        s += "#define FUSE_G " + std::to_string(G) + "\n#define FUSE_EPL " + std::to_string(EPL) +
             "\n#define FUSE_VEC " + std::to_string(VEC) + "\n#define FUSE_RS " + std::to_string(RS) +
             "\n#define FUSE_BLOCK " + std::to_string(BLOCK) + "\n#define FUSE_AGG " + std::to_string(ac) +
             "\n#define FUSE_WPR " + std::to_string(WPR) + "\n#define FUSE_LDSX " + std::to_string(ldsx) +
             "\n#define FUSE_NCOLS " + std::to_string(n) + "\n";
        s += side_tables(sides, nsides, prog.side_used);
        s += emit_row_body(prog);
        s += kSrcRowDense;
        g_last_source = s;
        return s;
    }, plan, g_err);
    if (rc)
        return rc;
    g_last_kernel = plan->kernel_name;
    if (!launch)
        return 0;

    Plan::Loaded fn;
    if ((rc = rt.load(*plan, fn, g_err)))
        return rc;
    const int64_t nroots = (int64_t)prog.roots.size();          // > 1: MAgg bodies, full aggregate only
    if (nroots > 1 && (ac != 1 || rk != KIND_V))
        return fail(FUSE_EDESC, "several results only as full aggregates of row-vector bodies");
    int64_t out_count = ac == 0 ? (prog.result_vec ? m * n : m) : ac == 1 ? nroots : ac == 2 ? m : n;
    if (rk == KIND_K)
        out_count = ac == 0 ? m * kd : ac == 3 ? kd : 1;
    else if (rk == KIND_VK)
        out_count = n * kd;
    if (m == 0 || n == 0)
        return zero_fill(fn, out, out_count, stream);

    const int NW = BLOCK / 64;
    const int64_t rows_per_iter = WPR > 1 ? RS : (int64_t)(64 / G) * RS * NW;
    const int cus = rt.num_cus();
    int64_t gx = (m + rows_per_iter - 1) / rows_per_iter;
    const int bpc = WPR > 1 ? std::max(1, 16 / WPR) : env_int("FUSE_ROW_BLOCKS_PER_CU", 2);
    const int64_t cap = std::max<int64_t>(1, (int64_t)cus * bpc / stripes);
    gx = std::min(gx, cap);
    Workspace ws;
    const int64_t nacc = rk == KIND_VK ? kd : 1;      // running sums per column
    size_t need = 64;
    if (ac == 3 && rk == KIND_K)
        need = (size_t)gx * (size_t)kd;
    else if (ac == 3)
        need = (size_t)gx * (size_t)(n * nacc);
    else if (ac == 1)
        need = (size_t)gx * stripes * (size_t)nroots;
    else if (ac == 2 && stripes > 1)
        need = (size_t)stripes * (size_t)m;
    if ((rc = rt.workspace(stream, need, ws, g_err)))
        return rc;

    fuse_kargs A;
    std::memset(&A, 0, sizeof A);
    A.x = X->data;
    A.m = m;
    A.n = n;
    A.ld = X->ld;
    A.out = out;
    A.partials = ws.partials;
    A.ticket = ws.ticket;
    fill_side_args(A, sides, nsides);
    if ((rc = rt.launch(fn.main, (unsigned)gx, (unsigned)stripes, BLOCK, stream, &A, sizeof A, g_err)))
        return rc;
    if (ac == 3 && rk != KIND_K)
        return run_combine(fn, ws.partials, (int)gx, (int)(n * nacc), out, stream);
    if (ac == 2 && stripes > 1)
        return run_combine(fn, ws.partials, stripes, (int)m, out, stream);
    return 0;
}

// ------------------------------------------------------------------ cell / magg --
// noalloc: the variant that may not allocate (fuse_magg_noalloc): the plan must be compiled and loaded
// already, only the flat form runs, and the block partials go to the library's fixed device array.
int cell_impl(const fuse_expr *exprs, int k, const fuse_dense *X, const fuse_side *sides, int nsides,
              int agg, double *out, void *stream_, bool launch, bool is_magg, bool noalloc = false)
{
    g_err.clear();
    Runtime &rt = Runtime::get();
    hipStream_t stream = (hipStream_t)stream_;
    if (!exprs)
        return fail(FUSE_EINVAL, "expr is NULL");
    if (k < 1 || k > FUSE_MAX_AGGS)
        return fail(FUSE_EINVAL, "k must be in [1, " + std::to_string(FUSE_MAX_AGGS) + "]");
    int rc = check_dense(X, "X", launch);
    if (rc)
        return rc;
    const int ac = agg_code(agg);
    if (ac < 0)
        return fail(FUSE_EINVAL, "unknown aggregation " + std::to_string(agg));
    const int64_t m = X->rows, n = X->cols;
    if (launch && !out && (ac == 1 ? k : ac == 0 ? m * n : ac == 2 ? m : n) > 0)
        return fail(FUSE_EINVAL, "out is NULL");
    Program prog;
    {
        // shape checks need to know which sides are used; parse first with kinds only
        if (nsides < 0 || nsides > FUSE_MAX_SIDES || (nsides > 0 && !sides))
            return fail(FUSE_EINVAL, "bad sides / nsides");
        for (int q = 0; q < nsides; ++q) {
            if (sides[q].kind == FUSE_SIDE_SPARSE)
                return fail(FUSE_EUNSUPPORTED, "side " + std::to_string(q) + ": sparse side inputs go with a CSR main input (fuse_cell_csr, fuse_magg_csr)");
            if (sides[q].kind < 0 || sides[q].kind > 3)
                return fail(FUSE_EINVAL, "side " + std::to_string(q) + ": unknown side kind");
        }
        rc = parse_cached(Tmpl::CELL, exprs, k, sides, nsides, prog, g_err);
        if (rc)
            return rc;
    }
    if ((rc = check_sides(sides, nsides, m, n, launch, prog.side_used)))
        return rc;

    // flat form: one contiguous index space
    bool flat = (ac == 0 || ac == 1) && (X->ld == n || m <= 1);
    for (int q = 0; q < nsides && flat; ++q)
        if (prog.side_used[q]) {
            if (sides[q].kind == FUSE_SIDE_MATRIX)
                flat = sides[q].m.ld == n || m <= 1;
            else if (sides[q].kind != FUSE_SIDE_SCALAR)
                flat = false;
        }
    if (!flat && noalloc)
        return fail(FUSE_EUNSUPPORTED, "fuse_magg_noalloc: only contiguous inputs (ld = cols) with matrix and scalar "
                                       "side inputs");
    if (!flat) {
        // 2-D form: the Cell body (or the k bodies of a MAgg) as a Row body without row aggregates
        Program rprog;
        if ((rc = parse_cached(Tmpl::ROW_DENSE, exprs, k, sides, nsides, rprog, g_err, true)))
            return rc;
        return row_dense_impl(rprog, rprog.key, X, sides, nsides, agg, out, stream, launch,
                              is_magg ? "fuse_magg2d" : "fuse_cell2d");
    }

    bool vec2 = !launch || aligned16(X->data);
    for (int q = 0; q < nsides && vec2; ++q)
        if (prog.side_used[q] && sides[q].kind == FUSE_SIDE_MATRIX)
            vec2 = !launch || aligned16(sides[q].m.data);
    if (ac == 0 && launch && !aligned16(out))
        vec2 = false;
    const int VEC = vec2 ? 2 : 1;
    int nmat = 1;
    for (int q = 0; q < nsides; ++q)
        nmat += prog.side_used[q] && sides[q].kind == FUSE_SIDE_MATRIX;
    int UNROLL = env_int("FUSE_CELL_UNROLL", 0);
    // vectors per thread and input in flight.  Measured (1e5 .. 1e6 x 1000): one input 8; two inputs 4 (X*Y full_agg
    // 225 us against 232 with 8, no_agg 424 against 441); three inputs and a full aggregate 8 (the 2.4 GB MAgg
    // workload 339 us against 348 with 4 and 352 with 16; sum(X*Y*Z) on 24 GB 3.39 against 3.45 ms)
    if (UNROLL <= 0)
        UNROLL = nmat <= 1 ? 8 : (nmat == 3 && ac == 1) ? 8 : (nmat <= 4 ? 4 : 2);
    // threads per block (FUSE_CELL_BLOCK: 256, 512 or 1024; 0 = by rule)
    int CBLOCK = env_int("FUSE_CELL_BLOCK", 0);
    if (CBLOCK != 256 && CBLOCK != 512 && CBLOCK != 1024)
        CBLOCK = 256;

    const std::string key = std::string(is_magg ? "magg|" : "cell|") + prog.key + "|" +
                            side_key(sides, nsides) + "|agg" + std::to_string(ac) + "|v" + std::to_string(VEC) +
                            "u" + std::to_string(UNROLL) + "b" + std::to_string(CBLOCK) + "nt" + std::to_string(env_int("FUSE_NT", 1));
    std::shared_ptr<Plan> plan;
    const char *not_ready = "fuse_magg_noalloc: this operator is not compiled and loaded on the current device yet; "
                            "call fuse_magg once with the same descriptor, side kinds and pointer alignment first";
    if (noalloc && !rt.find_plan(key, plan))
        return fail(FUSE_ENOTREADY, not_ready);
    rc = noalloc ? 0 : rt.plan(key, is_magg ? "fuse_magg" : "fuse_cell", [&](const std::string &name) {
        std::string s = kSrcArgs;
        s += "#define FUSE_NT " + std::to_string(env_int("FUSE_NT", 1)) + "\n";
        s += kSrcCommon;
        s += "#define FUSE_KERNEL_NAME " + name + "\n";
        s += "#define FUSE_K " + std::to_string(k) + "\n#define FUSE_VEC " + std::to_string(VEC) +
             "\n#define FUSE_UNROLL " + std::to_string(UNROLL) + "\n#define FUSE_BLOCK " + std::to_string(CBLOCK) +
             "\n#define FUSE_FULL " + std::to_string(ac == 1) + "\n";
        s += side_tables(sides, nsides, prog.side_used);
        s += "#define FUSE_SIDE_IS_MATRIX(k) (fuse_side_kind[k] == 0 && fuse_side_used[k])\n";
        s += emit_cell_body(prog);
        s += kSrcCell;
        g_last_source = s;
        return s;
    }, plan, g_err);
    if (rc)
        return rc;
    g_last_kernel = plan->kernel_name;
    if (!launch)
        return 0;

    Plan::Loaded fn;
    if (noalloc) {
        if (!rt.loaded(*plan, fn))
            return fail(FUSE_ENOTREADY, not_ready);
    } else if ((rc = rt.load(*plan, fn, g_err)))
        return rc;
    const int64_t N = m * n;
    if (N == 0)
        return zero_fill(fn, out, ac == 1 ? k : 0, stream);
    const int64_t nvec = N / VEC;
    const int cus = rt.num_cus();
    int64_t gx = std::max<int64_t>(nvec / ((int64_t)CBLOCK * UNROLL), (N + CBLOCK - 1) / CBLOCK > 4 ? 4 : 1);
    gx = std::max<int64_t>(1, std::min<int64_t>(gx, (int64_t)cus * env_int("FUSE_CELL_BLOCKS_PER_CU", 1)));
    // small inputs: the cost of finishing (one arrival ticket and one partial per block, summed by the last block)
    // grows with the number of blocks, so a block gets at least 128 KB to read (24 MB: 183 blocks, 11.4 us cold
    // against 12.2 us with 256 and 20 us with 1024; back to back from cache 5.9 against 6.5 us)
    if (ac == 1)
        gx = std::min<int64_t>(gx, std::max<int64_t>(16, N * 8 * nmat / (128 * 1024)));
    if (env_int("FUSE_CELL_GRID", 0) > 0)
        gx = env_int("FUSE_CELL_GRID", 0);
    Workspace ws;
    if (noalloc) {
        if ((size_t)gx * k > (size_t)FUSE_NOALLOC_MAX_PARTIALS)
            return fail(FUSE_EUNSUPPORTED, "fuse_magg_noalloc: " + std::to_string(gx) + " blocks x " + std::to_string(k) +
                                               " aggregates need more than the " + std::to_string(FUSE_NOALLOC_MAX_PARTIALS) +
                                               " block partials of the fixed workspace");
        if ((rc = noalloc_workspace(stream, ws, g_err)))
            return rc;
    } else if ((rc = rt.workspace(stream, (size_t)gx * k, ws, g_err)))
        return rc;
    fuse_kargs A;
    std::memset(&A, 0, sizeof A);
    A.x = X->data;
    A.m = m;
    A.n = n;
    A.ld = n;
    A.out = out;
    A.partials = ws.partials;
    A.ticket = ws.ticket;
    fill_side_args(A, sides, nsides);
    return rt.launch(fn.main, (unsigned)gx, 1, CBLOCK, stream, &A, sizeof A, g_err);
}

// ------------------------------------------------------------------------- row --
int row_csr_impl(const Program &prog, const fuse_csr *X, const fuse_side *sides, int nsides, int agg,
                 double *out, hipStream_t stream, bool launch, const char *name_prefix = "fuse_row_csr")
{
    Runtime &rt = Runtime::get();
    const int64_t m = X->rows, n = X->cols;
    const int ac = agg_code(agg);
    const int rk = prog.result_kind;
    const int kd = prog.kdim;
    if (rk == KIND_S && (ac == 2 || ac == 3))
        return fail(FUSE_EDESC, "row / column aggregation needs a row-vector result");
    if (rk == KIND_K && ac == 2)
        return fail(FUSE_EDESC, "a k-vector result has the variants no_agg, col_agg and full_agg");
    if (rk == KIND_VK && ac != 3)
        return fail(FUSE_EDESC, "an OUTERK result needs FUSE_AGG_COL / FUSE_AGG_COL_T");
    const int64_t nacck = rk == KIND_VK ? kd : 1;           // running sums per column

    // t(X) %*% f(X %*% V) over a matrix that stores a good part of its cells (Mnist-like: a quarter): the dense
    // matrix-unit form, whose LDS tile is filled from the CSR rows; its time does not depend on the density, the
    // lane-group form's is proportional to it (FUSE_MFMA_CSR_DENSITY: least stored share in percent, default 15;
    // FUSE_MFMA_CSR_MIN_K: least number of classes, default 5, 0 = never)
    {
        int vside = -1;
        const int min_k = env_int("FUSE_MFMA_CSR_MIN_K", 5);
        const double share = (m > 0 && n > 0) ? 100.0 * (double)X->nnz / ((double)m * (double)n) : 0.0;
        const int64_t tile_bytes = (16 * ((n + 15) / 16 * 16 + 1) + (int64_t)(4 + 2 + std::max(nsides, 1)) * 272 + 128) * 8;
        if (ac == 3 && min_k > 0 && kd >= min_k && n >= 16 && tile_bytes <= 158 * 1024 &&
            share >= (double)env_int("FUSE_MFMA_CSR_DENSITY", 15) && mfma_pattern(prog, sides, nsides, vside))
            return row_mfma_impl(prog, prog.key, nullptr, X, sides, nsides, vside, out, stream, launch);
    }

    // lanes per row (G) and register-resident cells per lane (C): C*G is the power of two that covers
    // the mean row length plus 1.5 standard deviations of a Poisson-like length (the few longer rows take
    // the strided tail loop); short rows use few lanes so that the group butterfly is paid once per C*G
    // cells.  Measured, 1e8 cells in 1000 columns: 10 per row 16 slots (32: slower), 100 per row 128
    // slots 217 us against 275 us with 256.
    int G = env_int("FUSE_CSR_G", 0);
    int C = env_int("FUSE_CSR_C", 0);
    if (G <= 0 || C <= 0) {
        const double avg = m > 0 ? (double)X->nnz / (double)m : 1.0;
        const int cover = next_pow2((int64_t)(avg + 1.5 * std::sqrt(avg) + 0.999));
        C = cover >= 4 ? 4 : cover;            // (4 cells = one 16-byte load of column indices; 2 per lane: 1.6x slower)
        G = std::min(64, std::max(1, cover / C));
        if (cover > 256)
            C = 4, G = 64;
    }
    const int RS = std::max(1, env_int("FUSE_CSR_RS", 1));
    const int BLOCK = std::max(64, env_int("FUSE_CSR_BLOCK", 1024));
    // Very short rows (a mean of up to 5.5 cells): the streaming skeleton, where a wave reads runs of
    // whole rows as contiguous cells.  Measured on 1000 columns, t(X)(Xv), 1e8 stored cells: 3 per row
    // 285 us against 500 us for lane groups, 10 per row 264 against 234; 5e7 stored cells: 4 per row
    // 135 against 157, 5 per row 132 against 144, 6 per row 126 against 119, 8 per row 124 against 115.
    // FUSE_CSR_STREAM: 0 never, 1 always, 2 by this rule.
    const int stream_mode = env_int("FUSE_CSR_STREAM", 2);
    const int SC = 4;                                    // cells per lane of the streaming skeleton (8: slower, 442 us on config 4)
    // bodies that never look at the row (no row aggregate, no per-row side, one value per cell)
    // run the streaming skeleton's flat form over the cell arrays, whatever the row lengths
    bool need_rid = prog.nred > 0 || ac == 2 || !prog.result_vec;
    for (int k = 0; k < nsides; ++k)
        need_rid |= prog.side_used[k] && (sides[k].kind == FUSE_SIDE_MATRIX || sides[k].kind == FUSE_SIDE_SPARSE || sides[k].kind == FUSE_SIDE_COLVEC);
    // (bodies with k-vectors run in the lane-group form only)
    const double mean_len = m > 0 ? (double)X->nnz / (double)m : 0.0;
    // LDS the streaming form needs per block beside column sums and staged row vectors: a histogram of
    // 64 * SC + 4 counters and 65 row totals per row aggregate, per wave
    const int64_t stream_fixed = (int64_t)(BLOCK / 64) * ((64 * SC + 4) * 4 + (int64_t)std::max(prog.nred, 1) * 65 * 8) + 2048;
    const bool streaming = kd == 0 && stream_fixed <= 120 * 1024 &&
                           (stream_mode == 1 || (stream_mode == 2 && (mean_len <= 5.5 || !need_rid)));

    // LDS plan: the column accumulator first, then staged row-vector sides if they fit
    int nrv = 0;
    for (int k = 0; k < nsides; ++k)
        nrv += prog.side_used[k] && sides[k].kind == FUSE_SIDE_ROWVEC;
    // one block per CU: most of the 160 KB of LDS can go to the column sums and the staged row vectors
    // (the streaming form keeps per-wave histograms and row totals there as well)
    const int64_t lds_budget = streaming ? std::min<int64_t>(96 * 1024, 156 * 1024 - stream_fixed) : 144 * 1024;
    // column sums: a per-block LDS vector while it fits, else fp64 atomics on the output
    const bool col_acc = ac == 3 && rk != KIND_K;          // per-column running sums (k per column for OUTERK)
    const bool cols_global = col_acc && n * nacck * 8 > lds_budget - 4096;
    const bool cols_lds = col_acc && !cols_global;
    const bool stage_rv = nrv > 0 && ((cols_lds ? n * nacck : 0) + (int64_t)nrv * n) * 8 <= lds_budget - 1024;
    const int64_t npad = (cols_lds || stage_rv) ? std::max<int64_t>(n, 1) : 1;
    const int64_t naccpad = cols_lds ? std::max<int64_t>(n * nacck, 1) : 1;

    // Sparse side inputs in the lane-group form: every group stages the column indices of the side's row in LDS
    // (FUSE_SCAP entries per group and side: 1.5 x the side's mean row length, a power of two, while it fits
    // beside the column sums and the staged row vectors); longer rows of a side are searched in memory.
    int nsparse = 0, scap = 0;
    if (!streaming) {
        double longest = 0.0;
        for (int k = 0; k < nsides; ++k)
            if (prog.side_used[k] && sides[k].kind == FUSE_SIDE_SPARSE && sides[k].sp) {
                ++nsparse;
                longest = std::max(longest, m > 0 ? (double)sides[k].sp->nnz / (double)m : 0.0);
            }
        if (nsparse > 0 && env_int("FUSE_CSR_SCAP", -1) != 0) {
            scap = std::min(1024, std::max(G, next_pow2((int64_t)(1.5 * longest + 8.0))));
            if (env_int("FUSE_CSR_SCAP", -1) > 0)
                scap = std::min(1024, next_pow2(env_int("FUSE_CSR_SCAP", -1)));
            const int64_t used = ((cols_lds ? naccpad : 0) + (stage_rv ? (int64_t)nrv * npad : 0)) * 8 + 8192;
            while (scap >= 8 && (int64_t)(BLOCK / G) * nsparse * scap * 4 > lds_budget - used)
                scap >>= 1;
            if (scap < 8)
                scap = 0;
        }
    }

    const int nt = env_int("FUSE_CSR_NT", streaming ? 1 : 0);
    // lane-group form: the rows are dealt to the blocks in pieces of FUSE_CSR_ILV steps of a block (default 1:
    // 256 rows with 16 rows per wave and 16 waves), round-robin, when every block gets at least four pieces;
    // otherwise (and with FUSE_CSR_ILV=0) every block takes one contiguous range balanced by rows + stored cells.
    // 1e7 x 1000, 1e8 stored cells, t(X)(Xv), medians of 6 x 20 calls: contiguous ranges 231.8 us, pieces of
    // 1 step 223.9, 2 steps 224.1, 8 steps 228.4; 1e6 x 1000 with a tenth stored 217 -> 202 us; 2e6 x 1000 with
    // 1 % stored and 2000 rows 70 % full 289 -> 246 us; 2e6 x 1000 with 20 cells per row 93 -> 87 us.
    int ilv = 0;
    if (!streaming) {
        const int ilv_env = env_int("FUSE_CSR_ILV", -1);          // set: taken as it is, also for small matrices
        ilv = ilv_env >= 0 ? ilv_env : 1;
        const int64_t rpi = (int64_t)(64 / G) * RS * (BLOCK / 64);
        const int64_t gx_est = std::max<int64_t>(1, std::min<int64_t>((m + rpi - 1) / rpi,
                                                                      (int64_t)rt.num_cus() * env_int("FUSE_CSR_BLOCKS_PER_CU", 1)));
        if (ilv_env < 0 && m < 4 * gx_est * ilv * rpi)
            ilv = 0;
    }
    const std::string key = std::string("rowcsr|") + prog.key + "|" + side_key(sides, nsides) + "|agg" +
                            std::to_string(ac) + (streaming ? "|stream" + std::to_string(SC) + "r" + std::to_string(need_rid)
                                                            : "|g" + std::to_string(G) + "c" + std::to_string(C) + "r" + std::to_string(RS)) + "b" +
                            std::to_string(BLOCK) + "p" + std::to_string(npad) + "a" + std::to_string(naccpad) + "s" + std::to_string(stage_rv) + (cols_global ? "G" : "") +
                            "w" + std::to_string(X->rowptr_is64 != 0) + std::to_string(m < (1LL << 30)) + "nt" +
                            std::to_string(nt) + "i" + std::to_string(ilv) + (scap ? "sp" + std::to_string(nsparse) + "x" + std::to_string(scap) : "");
    std::shared_ptr<Plan> plan;
    int rc = rt.plan(key, name_prefix, [&](const std::string &name) {
        std::string s = kSrcArgs;
        s += "#define FUSE_ILV " + std::to_string(ilv) + "\n";
        // group form: plain (cached) loads, the register slots of neighbouring rows overlap in
        // memory, so lines are re-used from cache; streaming form: every cell is read once
        s += "#define FUSE_NT " + std::to_string(nt) + "\n";
        s += kSrcCommon;
        s += "#define FUSE_KERNEL_NAME " + name + "\n";
        s += "#define FUSE_G " + std::to_string(G) + "\n#define FUSE_C " + std::to_string(streaming ? SC : C) +
             "\n#define FUSE_RS " + std::to_string(RS) + "\n#define FUSE_NEED_RID " + std::to_string(need_rid) +
             "\n#define FUSE_COLS_GLOBAL " + std::to_string(cols_global) +
             "\n#define FUSE_BLOCK " + std::to_string(BLOCK) + "\n#define FUSE_AGG " + std::to_string(ac) +
             "\n#define FUSE_RP64 " + std::to_string(X->rowptr_is64 != 0) + "\n#define FUSE_ROW32 " +
             std::to_string(m < (1LL << 30)) + "\n#define FUSE_NPAD " +
             std::to_string(npad) + "\n#define FUSE_NACCPAD " + std::to_string(naccpad) + "\n#define FUSE_STAGE_RV " + std::to_string(stage_rv) +
             "\n#define FUSE_NRV " + std::to_string(std::max(nrv, 1)) + "\n#define FUSE_NSPARSE " + std::to_string(std::max(nsparse, 1)) +
             "\n#define FUSE_SCAP " + std::to_string(scap) + "\n";
        s += side_tables(sides, nsides, prog.side_used);
        s += emit_row_body(prog);
        s += streaming ? kSrcRowCsrStream : kSrcRowCsr;
        g_last_source = s;
        return s;
    }, plan, g_err);
    if (rc)
        return rc;
    g_last_kernel = plan->kernel_name;
    if (!launch)
        return 0;

    Plan::Loaded fn;
    if ((rc = rt.load(*plan, fn, g_err)))
        return rc;
    int64_t out_count = ac == 0 ? (prog.result_vec ? X->nnz : m)
                                : ac == 1 ? (int64_t)prog.roots.size() : ac == 2 ? m : n;
    if (rk == KIND_K)
        out_count = ac == 0 ? m * kd : ac == 3 ? kd : 1;
    else if (rk == KIND_VK)
        out_count = n * kd;
    if (m == 0)
        return zero_fill(fn, out, out_count, stream);
    if (out_count == 0)                        // e.g. column sums of a matrix without columns: nothing to write
        return 0;

    const int cus = rt.num_cus();
    const int NW = BLOCK / 64;
    if (streaming && !need_rid && X->nnz == 0)
        return zero_fill(fn, out, ac == 0 ? 0 : out_count, stream);
    const int64_t rows_per_iter = streaming ? NW : (int64_t)(64 / G) * RS * NW;
    int64_t gx = (m + rows_per_iter - 1) / rows_per_iter;
    if (streaming && !need_rid)
        gx = (X->nnz + (int64_t)64 * SC * NW - 1) / ((int64_t)64 * SC * NW);
    gx = std::max<int64_t>(1, std::min<int64_t>(gx, (int64_t)cus * env_int("FUSE_CSR_BLOCKS_PER_CU", 1)));
    Workspace ws;
    const size_t need = cols_lds ? (size_t)gx * (size_t)(n * nacck)
                                 : (size_t)gx * std::max<size_t>(prog.roots.size(), (size_t)std::max(kd, 1));
    if (cols_global && (rc = zero_fill(fn, out, n * nacck, stream)))
        return rc;
    if ((rc = rt.workspace(stream, need, ws, g_err)))
        return rc;
    fuse_kargs A;
    std::memset(&A, 0, sizeof A);
    A.x = X->vals;
    A.colidx = X->colidx;
    A.rowptr = X->rowptr;
    A.m = m;
    A.n = n;
    A.nnz = X->nnz;
    if (X->nnz == 0) {
        // no stored cell at all: the kernel's (masked) loads still need a valid
        // address, so point them at one dummy cell inside the workspace
        A.x = ws.partials;
        A.colidx = reinterpret_cast<const int *>(ws.ticket) + 16;   // stays zero
        A.nnz = 1;
    }
    A.out = out;
    A.partials = ws.partials;
    A.ticket = ws.ticket;
    fill_side_args(A, sides, nsides);
    if ((rc = rt.launch(fn.main, (unsigned)gx, 1, BLOCK, stream, &A, sizeof A, g_err)))
        return rc;
    if (cols_lds)
        return run_combine(fn, ws.partials, (int)gx, (int)(n * nacck), out, stream);
    return 0;
}

// Cell / MAgg bodies over a CSR main input: the sparse-safe binding of the Cell
// template (Sec. 2.2 "Template Types").  A Cell body is a Row body without row
// aggregates, so it runs in the CSR Row skeleton; k > 1 results only with the
// full aggregate (MAgg).
int cell_csr_impl(const fuse_expr *exprs, int k, const fuse_csr *X, const fuse_side *sides, int nsides,
                  int agg, double *out, void *stream_, bool launch, bool is_magg)
{
    g_err.clear();
    if (!exprs)
        return fail(FUSE_EINVAL, "expr is NULL");
    if (k < 1 || k > FUSE_MAX_AGGS)
        return fail(FUSE_EINVAL, "k must be in [1, " + std::to_string(FUSE_MAX_AGGS) + "]");
    const int ac = agg_code(agg);
    if (ac < 0)
        return fail(FUSE_EINVAL, "unknown aggregation " + std::to_string(agg));
    int rc = check_csr(X, launch);
    if (rc)
        return rc;
    if (nsides < 0 || nsides > FUSE_MAX_SIDES || (nsides > 0 && !sides))
        return fail(FUSE_EINVAL, "bad sides / nsides");
    for (int q = 0; q < nsides; ++q)
        if (sides[q].kind < 0 || (sides[q].kind > 3 && sides[q].kind != FUSE_SIDE_SPARSE))
            return fail(FUSE_EINVAL, "side " + std::to_string(q) + ": unknown side kind");
    Program cprog, prog;
    if ((rc = parse_cached(Tmpl::CELL, exprs, k, sides, nsides, cprog, g_err)))     // Cell tokens only
        return rc;
    if ((rc = parse_cached(Tmpl::ROW_CSR, exprs, k, sides, nsides, prog, g_err)))   // kinds + sparse-safety
        return rc;
    if (!prog.result_vec)
        return fail(FUSE_EDESC, "not sparse-safe: the body does not depend on the main input");
    if ((rc = check_sides(sides, nsides, X->rows, X->cols, launch, prog.side_used, true)))
        return rc;
    const int64_t count = ac == 1 ? k : ac == 2 ? X->rows : ac == 3 ? X->cols : X->nnz;
    if (launch && !out && count > 0)
        return fail(FUSE_EINVAL, "out is NULL");
    return row_csr_impl(prog, X, sides, nsides, agg, out, (hipStream_t)stream_, launch,
                        is_magg ? "fuse_magg_csr" : "fuse_cell_csr");
}

int row_impl(const fuse_expr *expr, const fuse_dense *Xd, const fuse_csr *Xs, const fuse_side *sides,
             int nsides, int agg, double *out, void *stream_, bool launch, int64_t *count_only = nullptr)
{
    g_err.clear();
    hipStream_t stream = (hipStream_t)stream_;
    if (!expr)
        return fail(FUSE_EINVAL, "expr is NULL");
    if ((Xd != nullptr) == (Xs != nullptr))
        return fail(FUSE_EINVAL, "exactly one of Xd / Xs must be given");
    if (agg_code(agg) < 0)
        return fail(FUSE_EINVAL, "unknown aggregation " + std::to_string(agg));
    int rc = Xd ? check_dense(Xd, "Xd", launch) : check_csr(Xs, launch);
    if (rc)
        return rc;
    if (nsides < 0 || nsides > FUSE_MAX_SIDES || (nsides > 0 && !sides))
        return fail(FUSE_EINVAL, "bad sides / nsides");
    for (int q = 0; q < nsides; ++q)
        if (sides[q].kind < 0 || sides[q].kind > FUSE_SIDE_SPARSE)
            return fail(FUSE_EINVAL, "side " + std::to_string(q) + ": unknown side kind");
    Program prog;
    if ((rc = parse_cached(Xd ? Tmpl::ROW_DENSE : Tmpl::ROW_CSR, expr, 1, sides, nsides, prog, g_err)))
        return rc;
    const int64_t m = Xd ? Xd->rows : Xs->rows, n = Xd ? Xd->cols : Xs->cols;
    if ((rc = check_sides(sides, nsides, m, n, launch, prog.side_used, Xs != nullptr)))
        return rc;
    for (int q = 0; q < nsides; ++q)
        if (sides[q].kind == FUSE_SIDE_SPARSE && prog.side_used[q] && prog.kdim > 0)
            return fail(FUSE_EUNSUPPORTED, "side " + std::to_string(q) + ": sparse side inputs are not built for bodies with k-vectors");
    {
        const int ac = agg_code(agg);
        const int64_t cells = Xd ? m * n : Xs->nnz;
        int64_t count = ac == 1 ? 1 : ac == 2 ? m : ac == 3 ? n : (prog.result_vec ? cells : m);
        if (prog.result_kind == KIND_K)
            count = ac == 0 ? m * prog.kdim : ac == 3 ? prog.kdim : 1;
        else if (prog.result_kind == KIND_VK)
            count = n * prog.kdim;
        if (count_only) {               // fuse_row_out_count: the variant must still be one the body has
            const int rk = prog.result_kind;
            if (rk == KIND_S && (ac == 2 || ac == 3))
                return fail(FUSE_EDESC, "row / column aggregation needs a row-vector result");
            if (rk == KIND_K && ac == 2)
                return fail(FUSE_EDESC, "a k-vector result has the variants no_agg, col_agg and full_agg");
            if (rk == KIND_VK && ac != 3)
                return fail(FUSE_EDESC, "an OUTERK result needs FUSE_AGG_COL / FUSE_AGG_COL_T");
            *count_only = count;
            return 0;
        }
        if (launch && !out && count > 0)
            return fail(FUSE_EINVAL, "out is NULL");
    }
    if (Xd)
        return row_dense_impl(prog, prog.key, Xd, sides, nsides, agg, out, stream, launch,
                              "fuse_row_dense");
    return row_csr_impl(prog, Xs, sides, nsides, agg, out, stream, launch);
}

// ----------------------------------------------------------------------- outer --
// Layout of a prepared left_mm pattern (fuse_outer_left_prepare): column offsets of X (cols + 1, of the width of
// X's row offsets), the row of every cell by column (int32), the place of every such cell in X's arrays (as fp64,
// exact below 2^53), and the cells' values in that order; every part a whole number of 16-byte granules.
// Sizes in doubles.
struct LeftPattern {
    size_t ptr, row, perm, val;
    size_t bytes() const { return (ptr + row + perm + val) * 8; }
};
LeftPattern left_pattern_layout(const fuse_csr *X)
{
    auto dbl = [](size_t bytes) { return (bytes + 15) / 16 * 2; };
    LeftPattern l;
    l.ptr = dbl((size_t)(X->cols + 1) * (X->rowptr_is64 ? 8 : 4));
    l.row = dbl((size_t)X->nnz * 4);
    l.perm = dbl((size_t)X->nnz * 8);
    l.val = l.perm;
    return l;
}

// pattern: a prepared left_mm pattern of X (device), or nullptr
int outer_impl(const fuse_expr *expr, const fuse_csr *X, const fuse_dense *U, const fuse_dense *V,
               const fuse_side *sides, int nsides, int agg, double *out, void *stream_, bool launch,
               const void *pattern = nullptr, bool with_pattern = false)
{
    g_err.clear();
    Runtime &rt = Runtime::get();
    hipStream_t stream = (hipStream_t)stream_;
    if (!expr)
        return fail(FUSE_EINVAL, "expr is NULL");
    int rc = check_csr(X, launch);
    if (rc)
        return rc;
    if ((rc = check_dense(U, "U", launch)) || (rc = check_dense(V, "V", launch)))
        return rc;
    int mode;                      // 0 no_agg, 1 full_agg, 2 right_mm, 3 left_mm
    switch (agg) {
    case FUSE_AGG_NONE: mode = 0; break;
    case FUSE_AGG_FULL: mode = 1; break;
    case FUSE_AGG_RIGHT_MM: mode = 2; break;
    case FUSE_AGG_LEFT_MM: mode = 3; break;
    case FUSE_AGG_ROW:
    case FUSE_AGG_COL:
    case FUSE_AGG_COL_T:
        return fail(FUSE_EUNSUPPORTED, "Outer has the variants no_agg, full_agg, right_mm and left_mm");
    default:
        return fail(FUSE_EINVAL, "unknown aggregation " + std::to_string(agg));
    }
    const int64_t out_count = mode == 0 ? X->nnz : mode == 1 ? 1 : mode == 2 ? X->rows * U->cols
                                                                               : X->cols * U->cols;
    if (launch && !out && out_count > 0)
        return fail(FUSE_EINVAL, "out is NULL");
    if (U->rows != X->rows || V->rows != X->cols || U->cols != V->cols)
        return fail(FUSE_ESHAPE, "Outer needs U: rows(X) x r and V: cols(X) x r");
    const int64_t r = U->cols;
    if (r < 1 || r > 1024)
        return fail(FUSE_EUNSUPPORTED, "Outer rank must be in [1, 1024]");
    if (nsides < 0 || nsides > FUSE_MAX_SIDES || (nsides > 0 && !sides))
        return fail(FUSE_EINVAL, "bad sides / nsides");
    for (int q = 0; q < nsides; ++q) {
        if (sides[q].kind == FUSE_SIDE_SPARSE)
            return fail(FUSE_EUNSUPPORTED, "side " + std::to_string(q) + ": Outer binds to dense side inputs (Table 1)");
        if (sides[q].kind < 0 || sides[q].kind > 3)
            return fail(FUSE_EINVAL, "side " + std::to_string(q) + ": unknown side kind");
    }
    Program prog;
    if ((rc = parse_cached(Tmpl::OUTER, expr, 1, sides, nsides, prog, g_err)))
        return rc;
    if ((rc = check_sides(sides, nsides, X->rows, X->cols, launch, prog.side_used)))
        return rc;

    const bool vec2 = (r % 2 == 0) && (U->ld % 2 == 0) && (V->ld % 2 == 0) &&
                      (!launch || (aligned16(U->data) && aligned16(V->data)));
    const int VEC = vec2 ? 2 : 1;
    const int64_t nvec = (r + VEC - 1) / VEC;
    // lanes per inner product: least padding with at most 8 vectors per lane
    int G = env_int("FUSE_OUTER_G", 0);
    if (G <= 0) {
        double best = 1e30;
        for (int g = 1; g <= 64; g <<= 1) {
            const int64_t epl = (nvec + g - 1) / g;
            if (epl > 8)
                continue;
            const double waste = (double)(epl * g) / (double)nvec + 0.02 * g / 64.0 * 0;
            if (waste < best - 1e-12) {
                best = waste;
                G = g;
            }
        }
        if (G <= 0)
            G = 64;
    }
    const int EPL = (int)((nvec + G - 1) / G);
    int UNR = env_int("FUSE_OUTER_UNR", 0);
    if (UNR <= 0)
        UNR = EPL >= 7 ? 2 : (EPL >= 3 ? 4 : 8);
    UNR = std::min(UNR, G);
    while (G % UNR)
        --UNR;
    const int BLOCK = std::max(64, env_int("FUSE_OUTER_BLOCK", 256));
    bool need_col = false;
    for (int q = 0; q < nsides; ++q)
        need_col |= prog.side_used[q] && (sides[q].kind == FUSE_SIDE_MATRIX || sides[q].kind == FUSE_SIDE_ROWVEC);

    // Column panels of V: worth it when V overflows an L2 and a row still has a few cells per panel.
    // Measured on 1e5 x 1e5, 100 cells per row, rank 100 (V = 80 MB): 8 to 16 panels are best; more
    // panels raise the L2 hit rate of the V gathers but stream U once more per panel.
    // FUSE_OUTER_PANELS: 0 never, 1 by this heuristic, 2 always (tests: panels on small inputs).
    int npanels = 0, panel_w = 0;
    const int panel_mode = env_int("FUSE_OUTER_PANELS", 1);
    if (mode <= 1 && panel_mode != 0 && X->rows > 0 && X->cols > 0) {
        const bool force = panel_mode == 2;
        const int64_t vbytes = X->cols * V->ld * 8;
        const int64_t panel_bytes = (int64_t)std::max(1, env_int("FUSE_OUTER_PANEL_KB", 5120)) * 1024;
        if (force || vbytes > (int64_t)env_int("FUSE_OUTER_PANEL_MIN_KB", 4096) * 1024) {
            int64_t P = (vbytes + panel_bytes - 1) / panel_bytes;
            P = std::min<int64_t>((P + 7) / 8 * 8, 1024);
            const double per_row = (double)X->nnz / (double)X->rows;
            while (!force && P > 8 && per_row / (double)P < 2.0)
                P -= 8;
            const int64_t W = std::max<int64_t>(1, (X->cols + P - 1) / P);
            P = (X->cols + W - 1) / W;
            const int64_t pp_bytes = (P + 1) * X->rows * (X->rowptr_is64 ? 8 : 4);
            if ((force || per_row / (double)P >= 1.0) && P >= 2 && pp_bytes <= ((int64_t)1 << 30)) {
                npanels = (int)P;
                panel_w = (int)W;
            }
        }
    }
    const bool panels = npanels > 0;
    if (panels) {
        UNR = env_int("FUSE_OUTER_PANEL_UNR", 2);
        UNR = std::max(1, std::min(UNR, G));
        while (G % UNR)
            --UNR;
    }
    // U-stationary form (FUSE_OUTER_STATIONARY, default 1): one block of 8 waves per CU keeps its rows of U in LDS and
    // walks many small panels (FUSE_OUTER_SPANEL_KB of V each, default 4096) with them; taken when at least 64 rows of U
    // fit into the LDS of a CU beside the books.  Rows per block and round: what balances the rounds, at most 256.
    int stat_rcw = 0;                    // rows per block and round (0: another form)
    // threads of the one block per CU: 12 waves with one step of gathers in flight each (133 registers) -- config 5: 8 waves
    // with two steps 615 - 630 us, 12 waves with one 560 - 570, 16 waves with one (128 registers, no spills) 680; two steps
    // at 12 waves spill (680 us and more)
    int SBLOCK = env_int("FUSE_OUTER_SBLOCK", 768);
    if (SBLOCK != 512 && SBLOCK != 768 && SBLOCK != 1024)
        SBLOCK = 768;
    // Only where re-reading U per panel is what costs: with many cells per row and panel the streamed-U form with a lane
    // group per row (U_i in registers, 3 waves per SIMD) is the faster one -- 2e4 x 2e4, rank 100, a tenth of the cells
    // stored: 23 against 19.6 Gcells/s; a hundredth: 18 against 17 (FUSE_OUTER_STATIONARY: 0 never, 1 by this rule, 2 always).
    const int stat_mode = env_int("FUSE_OUTER_STATIONARY", 1);
    const bool stat_pays = panels && (double)X->nnz / (double)X->rows / (double)npanels <= 16.0;
    if (panels && stat_mode != 0 && (stat_mode == 2 || panel_mode == 2 || stat_pays)) {
        const int64_t up = nvec * VEC;
        const int64_t books = 3 * 256 * (4 + (X->rowptr_is64 ? 8 : 4)) + 3 * 4 * 4 + (SBLOCK / 64) * 8 + 32;   // all LDS beside the rows
        const int64_t cap = std::min<int64_t>(256, ((int64_t)160 * 1024 - books) / (up * 8));
        const int64_t blocks = rt.num_cus();
        if (cap >= 64) {
            const int64_t rounds = std::max<int64_t>(1, (X->rows + blocks * cap - 1) / (blocks * cap));
            int64_t rb = (X->rows + rounds * blocks - 1) / (rounds * blocks);
            if (env_int("FUSE_OUTER_RB", 0) > 0)
                rb = env_int("FUSE_OUTER_RB", 0);
            stat_rcw = (int)std::max<int64_t>(1, std::min<int64_t>(rb, cap));
            // many small panels: U costs nothing per panel here
            const int64_t vbytes = X->cols * V->ld * 8;
            const int64_t pbytes = (int64_t)std::max(1, env_int("FUSE_OUTER_SPANEL_KB", 4096)) * 1024;
            int64_t P = std::max<int64_t>(2, std::min<int64_t>(1024, (vbytes + pbytes - 1) / pbytes));
            if (panel_mode == 2)
                P = std::max<int64_t>(P, std::min<int64_t>(npanels, 1024));        // tests: tiny panels stay tiny
            const int64_t W = std::max<int64_t>(1, (X->cols + P - 1) / P);
            P = (X->cols + W - 1) / W;
            if (P >= 2 && (P + 1) * X->rows * (X->rowptr_is64 ? 8 : 4) <= ((int64_t)1 << 30)) {
                npanels = (int)P;
                panel_w = (int)W;
            } else {
                stat_rcw = 0;
            }
        }
    }
    // Flat form of the panel walk (FUSE_OUTER_FLAT, default 1): a wave takes RC rows at a time and deals their
    // cells inside the panel to its lane groups as one list; the chunk's U rows are staged in LDS.  RC: about 50
    // cells per chunk and panel (a round of the wave holds 64), a power of two <= 16; the staged rows of a block
    // (waves x RC x rank doubles) must fit in 60 KB.
    int flat_rc = 0;
    if (panels && !stat_rcw && env_int("FUSE_OUTER_FLAT", 1) != 0 &&
        (panel_mode == 2 || (double)X->nnz / (double)X->rows / (double)npanels <= 16.0)) {
        const double per_row_panel = (double)X->nnz / (double)X->rows / (double)npanels;
        int rc = env_int("FUSE_OUTER_RC", 0);
        if (rc <= 0) {
            rc = 1;
            while (rc < 16 && per_row_panel * (rc * 2) <= 56.0)
                rc <<= 1;
        }
        rc = std::min(16, next_pow2(rc));
        const int64_t up = nvec * VEC;                       // LDS pitch of a staged row of U
        while (rc > 1 && (int64_t)(BLOCK / 64) * rc * up * 8 > 60 * 1024)
            rc >>= 1;
        if ((int64_t)(BLOCK / 64) * rc * up * 8 <= 60 * 1024)
            flat_rc = rc;
    }

    // left_mm: by default over the transposed pattern of X (built per call in the workspace) as the right_mm
    // traversal with U and V exchanged; FUSE_OUTER_LEFT_TRANSPOSE=0 keeps the scatter with fp64 atomics
    if (with_pattern && (mode != 3 || X->rows > 2147483647LL / 16))
        return fail(FUSE_EUNSUPPORTED, "a prepared pattern serves left_mm of a matrix with fewer than 2^27 rows");
    if (with_pattern && launch && !pattern && X->nnz > 0)
        return fail(FUSE_EINVAL, "pattern is NULL");
    const bool transposed = with_pattern || (mode == 3 && env_int("FUSE_OUTER_LEFT_TRANSPOSE", 1) != 0 && X->rows <= 2147483647LL / 16);
    const int kmode = transposed ? 2 : mode;
    const bool out_vec = vec2 && (!launch || aligned16(out));
    const int flat_wpe = std::max(1, std::min(8, env_int("FUSE_OUTER_WPE", 2)));      // waves per SIMD the flat form is built for (3: spills, 898 against 810 us)
    const int KBLOCK = stat_rcw ? SBLOCK : BLOCK;                // threads per block of the main kernel
    int sunr = env_int("FUSE_OUTER_SUNR", SBLOCK > 512 ? 1 : 2);  // steps of a wave whose gathers leave together (stationary form)
    sunr = (sunr >= 2 && G % 2 == 0) ? 2 : 1;
    const int uq = std::max(1, std::min(16, env_int("FUSE_OUTER_UQ", 4)));      // vectors of U per thread in flight while the rows are staged
    const std::string key = std::string("outer|") + (panels ? (stat_rcw ? "stat" + std::to_string(stat_rcw) + "r" + std::to_string(r) + "u" + std::to_string(sunr) + "q" + std::to_string(uq) + "|"
                                                             : flat_rc ? "flat" + std::to_string(flat_rc) + "r" + std::to_string(r) + "w" + std::to_string(flat_wpe) + "|" : std::string("panels|")) : std::string("")) + prog.key + "|" + side_key(sides, nsides) + "|agg" +
                            std::to_string(kmode) + (transposed ? "T" : "") + (kmode == 2 && out_vec ? "o" : "") + "|v" + std::to_string(VEC) + "g" + std::to_string(G) + "e" +
                            std::to_string(EPL) + "u" + std::to_string(UNR) + "b" + std::to_string(KBLOCK) + "w" +
                            std::to_string(X->rowptr_is64 != 0);
    std::shared_ptr<Plan> plan;
    rc = rt.plan(key, "fuse_outer", [&](const std::string &name) {
        std::string s = kSrcArgs;
        s += "#define FUSE_NT 0\n";
        s += kSrcCommon;
        s += "#define FUSE_KERNEL_NAME " + name + "\n";
        s += "#define FUSE_G " + std::to_string(G) + "\n#define FUSE_EPL " + std::to_string(EPL) +
             "\n#define FUSE_VEC " + std::to_string(VEC) + "\n#define FUSE_UNR " + std::to_string(UNR) +
             "\n#define FUSE_BLOCK " + std::to_string(KBLOCK) + "\n#define FUSE_MODE " +
             std::to_string(kmode) + "\n#define FUSE_TRANSPOSED " + std::to_string(transposed) + "\n#define FUSE_OUT_VEC " + std::to_string(out_vec) + "\n#define FUSE_RP64 " + std::to_string(X->rowptr_is64 != 0) +
             "\n#define FUSE_NEED_COL " + std::to_string(need_col) + "\n#define FUSE_PANELS " + std::to_string(panels ? (stat_rcw ? 3 : flat_rc ? 2 : 1) : 0) +
             "\n#define FUSE_RANK " + std::to_string(r) + "\n#define FUSE_RC " + std::to_string(std::max(flat_rc, 1)) +
             "\n#define FUSE_RB " + std::to_string(std::max(stat_rcw, 1)) + "\n#define FUSE_SUNR " + std::to_string(sunr) +
             "\n#define FUSE_WPE " + std::to_string(stat_rcw ? SBLOCK / 256 : flat_wpe) + "\n#define FUSE_UQ " + std::to_string(uq) + "\n";
        s += side_tables(sides, nsides, prog.side_used);
        s += emit_outer_body(prog);
        s += kSrcOuter;
        g_last_source = s;
        return s;
    }, plan, g_err);
    if (rc)
        return rc;
    g_last_kernel = plan->kernel_name;
    if (!launch)
        return 0;

    Plan::Loaded fn;
    if ((rc = rt.load(*plan, fn, g_err)))
        return rc;
    if (X->rows == 0 || X->nnz == 0)
        return zero_fill(fn, out, mode == 0 ? 0 : out_count, stream);
    if (mode == 3 && !transposed && (rc = zero_fill(fn, out, out_count, stream)))
        return rc;
    const int cus = rt.num_cus();
    const int NW = BLOCK / 64;
    int64_t gx = ((transposed ? X->cols : X->rows) + NW - 1) / NW;
    gx = std::max<int64_t>(1, std::min<int64_t>(gx, (int64_t)cus * env_int("FUSE_OUTER_BLOCKS_PER_CU", 8)));
    size_t pp_doubles = 0;
    if (panels) {
        // every block must be resident from the start: blocks that start late walk the panels out of
        // step with their XCD and evict the panel the others are using
        int bpc = env_int("FUSE_OUTER_PANEL_BLOCKS_PER_CU", 0);
        if (bpc <= 0)
            bpc = stat_rcw ? 1 : rt.resident_blocks_per_cu(fn.main, KBLOCK);
        gx = std::max<int64_t>(8, (int64_t)cus * bpc / 8 * 8);
        pp_doubles = (size_t)(npanels + 1) * (size_t)X->rows * (X->rowptr_is64 ? 8 : 4) / 8 + 1;
    }
    const size_t part_doubles = ((size_t)gx + 15) / 16 * 16;
    // transposed matrix: scratch of the counting sort, column offsets, row and value of every cell
    const size_t rpb = X->rowptr_is64 ? 8 : 4;
    auto dbl = [](size_t bytes) { return (bytes + 15) / 16 * 2; };           // doubles, 16-byte granules
    const size_t t_scratch = transposed ? dbl(transpose_scratch_bytes(X->rows, X->cols, X->nnz, X->rowptr_is64)) : 0,
                 t_ptr = dbl((size_t)(X->cols + 1) * rpb), t_row = dbl((size_t)X->nnz * 4),
                 t_val = (size_t)X->nnz;
    if (transposed)
        pp_doubles = with_pattern ? 0 : t_scratch + t_ptr + t_row + t_val;
    Workspace ws;
    if ((rc = rt.workspace(stream, part_doubles + pp_doubles, ws, g_err)))
        return rc;
    fuse_kargs A;
    std::memset(&A, 0, sizeof A);
    A.x = X->vals;
    A.colidx = X->colidx;
    A.rowptr = X->rowptr;
    A.m = X->rows;
    A.n = X->cols;
    A.nnz = X->nnz;
    A.u = U->data;
    A.v = V->data;
    A.ldu = U->ld;
    A.ldv = V->ld;
    A.rank = (int)r;
    A.out = out;
    A.partials = ws.partials;
    A.ticket = ws.ticket;
    fill_side_args(A, sides, nsides);
    if (with_pattern) {
        // the prepared pattern: nothing is sorted here
        const LeftPattern lp = left_pattern_layout(X);
        const double *base = static_cast<const double *>(pattern);
        A.x = base + lp.ptr + lp.row + lp.perm;
        A.rowptr = base;
        A.colidx = reinterpret_cast<const int *>(base + lp.ptr);
        A.m = X->cols;
        A.n = X->rows;
        A.u = V->data;
        A.v = U->data;
        A.ldu = V->ld;
        A.ldv = U->ld;
    } else if (transposed) {
        double *base = ws.partials + part_doubles;
        void *scratch = base, *tptr = base + t_scratch;
        int *trow = reinterpret_cast<int *>(base + t_scratch + t_ptr);
        double *tval = base + t_scratch + t_ptr + t_row;
        if (transpose_launch(X->rowptr, X->rowptr_is64, X->colidx, X->vals, X->rows, X->cols, X->nnz, scratch, tptr,
                             trow, tval, stream))
            return fail(FUSE_ERUNTIME, "left_mm: launching the pattern transposition failed");
        A.x = tval;
        A.colidx = trow;
        A.rowptr = tptr;
        A.m = X->cols;
        A.n = X->rows;
        A.u = V->data;
        A.v = U->data;
        A.ldu = V->ld;
        A.ldv = U->ld;
    }
    if (panels) {
        if (!fn.prep)
            return fail(FUSE_ERUNTIME, "panel plan without its preparatory kernel");
        A.npanels = npanels;
        A.panel_w = panel_w;
        A.panel_ptr = ws.partials + part_doubles;
        const int64_t gp = (X->rows * 16 + 255) / 256;                 // 16 lanes per row
        if ((rc = rt.launch(fn.prep, (unsigned)gp, 1, 256, stream, &A, sizeof A, g_err)))
            return rc;
    }
    return rt.launch(fn.main, (unsigned)gx, 1, KBLOCK, stream, &A, sizeof A, g_err);
}

// values_only: the pattern exists, only the values of X are brought into its order again
int outer_left_prepare_impl(const fuse_csr *X, void *pattern, void *stream_, bool values_only)
{
    g_err.clear();
    int rc = check_csr(X, true);
    if (rc)
        return rc;
    if (X->rows > 2147483647LL / 16)
        return fail(FUSE_EUNSUPPORTED, "a prepared pattern serves left_mm of a matrix with fewer than 2^27 rows");
    if (X->rows == 0 || X->cols == 0 || X->nnz == 0)
        return 0;                              // calls with such a matrix never look at the pattern
    if (!pattern)
        return fail(FUSE_EINVAL, "pattern is NULL");
    if (reinterpret_cast<uintptr_t>(pattern) & 15u)
        return fail(FUSE_EINVAL, "pattern must be 16-byte aligned");
    hipStream_t stream = (hipStream_t)stream_;
    const LeftPattern lp = left_pattern_layout(X);
    if (values_only) {
        double *b = static_cast<double *>(pattern);
        if (gather_launch(b + lp.ptr + lp.row + lp.perm, X->vals, b + lp.ptr + lp.row, X->nnz, stream))
            return fail(FUSE_ERUNTIME, "fuse_outer_left_values: launch failed");
        return 0;
    }
    const size_t scratch = (transpose_scratch_bytes(X->rows, X->cols, X->nnz, X->rowptr_is64) + 15) / 16 * 2;
    Workspace ws;
    if ((rc = Runtime::get().workspace(stream, 64 + scratch + (size_t)X->nnz, ws, g_err)))
        return rc;
    double *base = static_cast<double *>(pattern);
    double *iota = ws.partials + 64 + scratch;
    if (iota_launch(iota, X->nnz, stream) ||
        transpose_launch(X->rowptr, X->rowptr_is64, X->colidx, iota, X->rows, X->cols, X->nnz, ws.partials + 64, base,
                         reinterpret_cast<int *>(base + lp.ptr), base + lp.ptr + lp.row, stream))
        return fail(FUSE_ERUNTIME, "fuse_outer_left_prepare: launching the pattern transposition failed");
    if (gather_launch(base + lp.ptr + lp.row + lp.perm, X->vals, base + lp.ptr + lp.row, X->nnz, stream))
        return fail(FUSE_ERUNTIME, "fuse_outer_left_prepare: launch failed");
    return 0;
}

int check_csr_device(const fuse_csr *X, void *stream_)
{
    g_err.clear();
    int rc = check_csr(X, true);
    if (rc)
        return rc;
    hipStream_t stream = (hipStream_t)stream_;
    unsigned long long *dev = nullptr;
    unsigned long long bad[4] = {~0ull, ~0ull, ~0ull, 0ull};
    hipError_t e = hipMalloc((void **)&dev, sizeof bad);
    if (e != hipSuccess)
        return fail(FUSE_ENOMEM, std::string("fuse_check_csr: ") + hipGetErrorString(e));
    e = hipMemcpyAsync(dev, bad, sizeof bad, hipMemcpyHostToDevice, stream);
    if (e == hipSuccess && check_csr_launch(X->rowptr, X->rowptr_is64, X->colidx, X->rows, X->cols, X->nnz, dev, stream))
        e = hipErrorLaunchFailure;
    if (e == hipSuccess)
        e = hipMemcpyAsync(bad, dev, sizeof bad, hipMemcpyDeviceToHost, stream);
    if (e == hipSuccess)
        e = hipStreamSynchronize(stream);
    (void)hipFree(dev);
    if (e != hipSuccess)
        return fail(FUSE_ERUNTIME, std::string("fuse_check_csr: ") + hipGetErrorString(e));
    if (bad[3] & 1)
        return fail(FUSE_ESHAPE, "X: rowptr[0] is not 0");
    if (bad[0] != ~0ull)
        return fail(FUSE_ESHAPE, "X: row offsets decrease or leave [0, nnz] at row " + std::to_string(bad[0]));
    if (bad[3] & 2)
        return fail(FUSE_ESHAPE, "X: rowptr[rows] differs from nnz");
    if (bad[1] != ~0ull)
        return fail(FUSE_ESHAPE, "X: column index outside [0, cols) in row " + std::to_string(bad[1]));
    if (bad[2] != ~0ull)
        return fail(FUSE_ESHAPE, "X: column indices not strictly ascending in row " + std::to_string(bad[2]));
    return 0;
}

// No C++ exception may cross the C boundary.
template <typename F>
int guarded(F f)
{
    try {
        return f();
    } catch (const std::bad_alloc &) {
        return fail(FUSE_ENOMEM, "out of host memory");
    } catch (const std::exception &ex) {
        return fail(FUSE_ERUNTIME, std::string("internal error: ") + ex.what());
    }
}

}  // namespace

// =============================================================================
extern "C" {

int fuse_cell(const fuse_expr *expr, const fuse_dense *X, const fuse_side *sides, int nsides, int agg,
              double *out, void *stream)
{
    return guarded([&] { return cell_impl(expr, 1, X, sides, nsides, agg, out, stream, true, false); });
}

int fuse_magg(const fuse_expr *exprs, int k, const fuse_dense *X, const fuse_side *sides, int nsides,
              double *out_k, void *stream)
{
    return guarded([&] { return cell_impl(exprs, k, X, sides, nsides, FUSE_AGG_FULL, out_k, stream, true, true); });
}

int fuse_magg_noalloc(const fuse_expr *exprs, int k, const fuse_dense *X, const fuse_side *sides, int nsides,
                      double *out_k, void *stream)
{
    return guarded([&] { return cell_impl(exprs, k, X, sides, nsides, FUSE_AGG_FULL, out_k, stream, true, true, true); });
}

int fuse_row(const fuse_expr *expr, const fuse_dense *Xd, const fuse_csr *Xs, const fuse_side *sides,
             int nsides, int agg, double *out, void *stream)
{
    return guarded([&] { return row_impl(expr, Xd, Xs, sides, nsides, agg, out, stream, true); });
}

int fuse_outer(const fuse_expr *expr, const fuse_csr *X, const fuse_dense *U, const fuse_dense *V,
               const fuse_side *sides, int nsides, int agg, double *out, void *stream)
{
    return guarded([&] { return outer_impl(expr, X, U, V, sides, nsides, agg, out, stream, true); });
}

size_t fuse_outer_left_pattern_bytes(const fuse_csr *X)
{
    if (!X || X->rows < 0 || X->cols < 0 || X->nnz < 0)
        return 0;
    return left_pattern_layout(X).bytes();
}

int fuse_outer_left_prepare(const fuse_csr *X, void *pattern, void *stream)
{
    return guarded([&] { return outer_left_prepare_impl(X, pattern, stream, false); });
}

int fuse_outer_left_values(const fuse_csr *X, void *pattern, void *stream)
{
    return guarded([&] { return outer_left_prepare_impl(X, pattern, stream, true); });
}

int fuse_outer_left(const fuse_expr *expr, const fuse_csr *X, const void *pattern, const fuse_dense *U,
                    const fuse_dense *V, const fuse_side *sides, int nsides, double *out, void *stream)
{
    return guarded([&] { return outer_impl(expr, X, U, V, sides, nsides, FUSE_AGG_LEFT_MM, out, stream, true, pattern, true); });
}

int fuse_cell_csr(const fuse_expr *expr, const fuse_csr *X, const fuse_side *sides, int nsides, int agg,
                  double *out, void *stream)
{
    return guarded([&] { return cell_csr_impl(expr, 1, X, sides, nsides, agg, out, stream, true, false); });
}

int fuse_magg_csr(const fuse_expr *exprs, int k, const fuse_csr *X, const fuse_side *sides, int nsides,
                  double *out_k, void *stream)
{
    return guarded([&] { return cell_csr_impl(exprs, k, X, sides, nsides, FUSE_AGG_FULL, out_k, stream, true, true); });
}

int fuse_prepare_cell_csr(const fuse_expr *expr, const fuse_csr *X, const fuse_side *sides, int nsides, int agg)
{
    return guarded([&] { return cell_csr_impl(expr, 1, X, sides, nsides, agg, nullptr, nullptr, false, false); });
}

int fuse_prepare_magg_csr(const fuse_expr *exprs, int k, const fuse_csr *X, const fuse_side *sides, int nsides)
{
    return guarded([&] { return cell_csr_impl(exprs, k, X, sides, nsides, FUSE_AGG_FULL, nullptr, nullptr, false, true); });
}

int fuse_prepare_cell(const fuse_expr *expr, const fuse_dense *X, const fuse_side *sides, int nsides, int agg)
{
    return guarded([&] { return cell_impl(expr, 1, X, sides, nsides, agg, nullptr, nullptr, false, false); });
}

int fuse_prepare_magg(const fuse_expr *exprs, int k, const fuse_dense *X, const fuse_side *sides, int nsides)
{
    return guarded([&] { return cell_impl(exprs, k, X, sides, nsides, FUSE_AGG_FULL, nullptr, nullptr, false, true); });
}

int fuse_prepare_row(const fuse_expr *expr, const fuse_dense *Xd, const fuse_csr *Xs, const fuse_side *sides,
                     int nsides, int agg)
{
    return guarded([&] { return row_impl(expr, Xd, Xs, sides, nsides, agg, nullptr, nullptr, false); });
}

int fuse_row_out_count(const fuse_expr *expr, const fuse_dense *Xd, const fuse_csr *Xs, const fuse_side *sides,
                       int nsides, int agg, int64_t *count)
{
    if (!count)
        return guarded([&] { g_err.clear(); return fail(FUSE_EINVAL, "count is NULL"); });
    return guarded([&] { return row_impl(expr, Xd, Xs, sides, nsides, agg, nullptr, nullptr, false, count); });
}

int fuse_prepare_outer(const fuse_expr *expr, const fuse_csr *X, const fuse_dense *U, const fuse_dense *V,
                       const fuse_side *sides, int nsides, int agg)
{
    return guarded([&] { return outer_impl(expr, X, U, V, sides, nsides, agg, nullptr, nullptr, false); });
}

int fuse_check_csr(const fuse_csr *X, void *stream)
{
    return guarded([&] { return check_csr_device(X, stream); });
}

const char *fuse_last_error(void) { return g_err.c_str(); }

int fuse_cache_stats(int64_t *hits, int64_t *misses, double *compile_ms)
{
    fuse::Runtime::get().stats(hits, misses, compile_ms);
    return FUSE_OK;
}

int64_t fuse_cache_disk_hits(void)
{
    return fuse::Runtime::get().disk_hits();
}

void fuse_cache_clear(void)
{
    fuse::Runtime::get().clear();
    std::lock_guard<std::mutex> lk(g_parse_mu);
    g_parsed.clear();
}

size_t fuse_last_source(char *buf, size_t buflen)
{
    if (buf && buflen) {
        const size_t n = std::min(buflen - 1, g_last_source.size());
        std::memcpy(buf, g_last_source.data(), n);
        buf[n] = '\0';
    }
    return g_last_source.size();
}

const char *fuse_last_kernel(void) { return g_last_kernel.c_str(); }

}  // extern "C"
