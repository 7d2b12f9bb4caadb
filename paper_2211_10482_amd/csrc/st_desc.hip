// Descriptor-driven structures: from a textual unique set / redundancy map to generated kernels.
//
// The paper gives every tensor a unique set T_U (a product of comparisons over its index variables)
// and a redundancy map T_R, and generates code from them: index variables are ordered as written,
// each variable ranges from the maximum of its lower bounds to the minimum of its upper bounds, one
// loop nest per product term, and the same procedure over T_R reconstructs the redundant part (code
// generation section).  This file does that at run time for a descriptor given as text:
//
//   unique set   "T(i,j,k): (0<=i<n)*(i<=j<n)*(j<=k<n)"      factors: chained comparisons of affine
//                "B(i,j,l): (0<=i<n)*(i-w<=j<=i+w)*(0<=l<m)"  expressions over the variables, named
//                "D(i,j):   (0<=i<n)*(i=j)"                   parameters and integers
//   redundancy   "(0<=j<i<n) -> (j,i)"   terms "condition -> unique index", separated by ';', or the
//                word "sort" (every permutation of a stored tuple holds the same value)
//
// parse -> constraints  c*x_v + rest >= 0 | = 0,  attached to the LAST variable they mention (unit
// coefficient there), i.e. a lower or an upper bound of that variable in terms of earlier ones ->
// the loop nest (st_desc_nest) -> packed layout = visiting order of that nest -> host tables (start
// of the innermost run of every index prefix) -> HIP source specialised to the descriptor (bounds
// and sizes are literals) -> hiprtc -> module.  The generated kernels iterate runs of the unique set
// (one wave per run, lanes along the last variable), never the bounding box with a mask; only the
// reconstruction visits every dense element, as Property 5 requires.
#include <hip/hiprtc.h>

#include <algorithm>
#include <cctype>
#include <cstdio>
#include <cstring>
#include <map>
#include <mutex>
#include <string>
#include <vector>

#include "st_common.h"

namespace st {
namespace {

typedef int64_t i64;
constexpr int MAXD = 4;

// affine expression: constant + sum coef[name] * name
struct Affine {
    i64 c = 0;
    std::map<std::string, i64> t;
    void add(const Affine &o, i64 s)
    {
        c += s * o.c;
        for (auto &kv : o.t) {
            t[kv.first] += s * kv.second;
            if (t[kv.first] == 0) t.erase(kv.first);
        }
    }
};

struct Parser {
    const char *p;
    bool ok = true;
    explicit Parser(const char *s) : p(s) {}
    void ws() { while (*p && isspace((unsigned char)*p)) ++p; }
    bool eat(char ch) { ws(); if (*p == ch) { ++p; return true; } return false; }
    bool peek(char ch) { ws(); return *p == ch; }
    std::string ident()
    {
        ws();
        std::string s;
        if (isalpha((unsigned char)*p) || *p == '_')
            while (isalnum((unsigned char)*p) || *p == '_') s += *p++;
        return s;
    }
    bool integer(i64 &v)
    {
        ws();
        if (!isdigit((unsigned char)*p)) return false;
        v = 0;
        while (isdigit((unsigned char)*p)) { v = v * 10 + (*p - '0'); if (v > (i64)1 << 40) ok = false; ++p; }
        return true;
    }
    // term := [int '*'] ident | int
    bool term(Affine &out, i64 sign)
    {
        i64 v;
        if (integer(v)) {
            if (eat('*')) {
                std::string id = ident();
                if (id.empty()) return false;
                out.t[id] += sign * v;
                if (out.t[id] == 0) out.t.erase(id);
            } else out.c += sign * v;
            return true;
        }
        std::string id = ident();
        if (id.empty()) return false;
        out.t[id] += sign;
        if (out.t[id] == 0) out.t.erase(id);
        return true;
    }
    bool expr(Affine &out)
    {
        i64 sign = 1;
        ws();
        if (*p == '-') { sign = -1; ++p; } else if (*p == '+') ++p;
        if (!term(out, sign)) return false;
        for (;;) {
            ws();
            if (*p == '+') { ++p; if (!term(out, 1)) return false; }
            else if (*p == '-' && p[1] != '>') { ++p; if (!term(out, -1)) return false; }
            else return true;
        }
    }
    // relation: 0 none, 1 <=, 2 <, 3 =, 4 >=, 5 >
    int rel()
    {
        ws();
        if (p[0] == '<' && p[1] == '=') { p += 2; return 1; }
        if (p[0] == '>' && p[1] == '=') { p += 2; return 4; }
        if (p[0] == '=' && p[1] == '=') { p += 2; return 3; }
        if (p[0] == '<') { ++p; return 2; }
        if (p[0] == '>') { ++p; return 5; }
        if (p[0] == '=') { ++p; return 3; }
        return 0;
    }
};

// E >= 0 (eq = false) or E == 0 (eq = true)
struct Constraint { Affine e; bool eq; };

// '(' expr rel expr [rel expr ...] ')' appended to out
bool parse_factor(Parser &ps, std::vector<Constraint> &out)
{
    if (!ps.eat('(')) return false;
    Affine left;
    if (!ps.expr(left)) return false;
    int n = 0;
    for (;;) {
        int r = ps.rel();
        if (r == 0) break;
        Affine right;
        if (!ps.expr(right)) return false;
        Constraint c;
        c.eq = (r == 3);
        if (r == 1 || r == 2 || r == 3) { c.e.add(right, 1); c.e.add(left, -1); }   // right - left >= 0
        else { c.e.add(left, 1); c.e.add(right, -1); }                               // left - right >= 0
        if (r == 2 || r == 5) c.e.c -= 1;                                            // strict
        out.push_back(c);
        left = right;
        ++n;
    }
    return n > 0 && ps.eat(')');
}

bool parse_product(Parser &ps, std::vector<Constraint> &out)
{
    if (!parse_factor(ps, out)) return false;
    while (ps.eat('*'))
        if (!parse_factor(ps, out)) return false;
    return true;
}

// bound of a variable in terms of earlier variables: value = c + sum coef[u] * x_u
struct Bound { i64 c; i64 coef[MAXD]; };

struct RedTerm { std::vector<Bound> cond; /* each: expression >= 0 over all variables */ Bound map[MAXD]; };

std::string bound_text(const Bound &b, const std::vector<std::string> &vars, int nv)
{
    std::string s;
    char buf[64];
    for (int u = 0; u < nv; ++u) {
        if (b.coef[u] == 0) continue;
        if (b.coef[u] == 1) snprintf(buf, sizeof buf, "%s%s", s.empty() ? "" : " + ", vars[u].c_str());
        else if (b.coef[u] == -1) snprintf(buf, sizeof buf, "%s%s", s.empty() ? "-" : " - ", vars[u].c_str());
        else snprintf(buf, sizeof buf, "%s%lld*%s", s.empty() ? "" : " + ", (long long)b.coef[u], vars[u].c_str());
        s += buf;
    }
    if (b.c != 0 || s.empty()) {
        if (s.empty()) snprintf(buf, sizeof buf, "%lld", (long long)b.c);
        else snprintf(buf, sizeof buf, " %c %lld", b.c < 0 ? '-' : '+', (long long)(b.c < 0 ? -b.c : b.c));
        s += buf;
    }
    return s;
}

// the same as a C expression over x0..x{nv-1}
std::string bound_code(const Bound &b, int nv)
{
    std::string s = "(" + std::to_string((long long)b.c);
    for (int u = 0; u < nv; ++u)
        if (b.coef[u] != 0) s += " + (" + std::to_string((long long)b.coef[u]) + ") * x" + std::to_string(u);
    return s + ")";
}

i64 bound_eval(const Bound &b, const i64 *x, int nv)
{
    i64 v = b.c;
    for (int u = 0; u < nv; ++u) v += b.coef[u] * x[u];
    return v;
}

}  // namespace

struct Desc {
    int d = 0;
    std::string name;
    std::vector<std::string> vars;
    i64 dims[MAXD] = {0, 0, 0, 0};
    i64 first[MAXD] = {0, 0, 0, 0}, last[MAXD] = {0, 0, 0, 0};   // constant part of every variable's range
    bool first_implied[MAXD] = {false, false, false, false};    // some other lower bound never falls below `first`
    bool last_implied[MAXD] = {false, false, false, false};     // some other upper bound never exceeds `last`
    std::vector<Bound> lo[MAXD], hi[MAXD];       // x_v >= each lo, x_v <= each hi (over x_0..x_{v-1})
    bool empty = false;                          // a constraint on the parameters alone is false
    bool red_sort = false;
    std::vector<RedTerm> red;
    i64 count = 0, prefixes = 1;
    std::vector<int32_t> table;                  // [prefixes] run start or -1, then [nruns] prefix ids
    i64 nruns = 0;
    // moment kernels (order 2 or 3, equal extents n <= 256): blocks of `mbs` indices, `ntiles` block tuples
    // that hold at least one unique entry; their block coordinates follow the run list in the table
    i64 mbs = 0, ntiles = 0, mnp = 0;
    std::string nest, source;
    std::mutex mu;
    struct Loaded { hipModule_t mod; hipFunction_t fn[10]; };  // list, thp, expand, gather, moment, moment_reduce, mttkrp, mttkrp_combine, sum_last, expand_onto
    std::map<int, Loaded> modules;               // per device
    std::string error;
};

namespace {

bool to_bound(const Affine &e, const Desc &D, const std::map<std::string, i64> &params, Bound &b, std::string &err)
{
    b.c = e.c;
    for (int u = 0; u < MAXD; ++u) b.coef[u] = 0;
    for (auto &kv : e.t) {
        auto it = std::find(D.vars.begin(), D.vars.end(), kv.first);
        if (it != D.vars.end()) b.coef[it - D.vars.begin()] += kv.second;
        else {
            auto pit = params.find(kv.first);
            if (pit == params.end()) { err = "unknown name '" + kv.first + "'"; return false; }
            b.c += kv.second * pit->second;
        }
    }
    return true;
}

// attach  E >= 0 / E == 0  to the last variable it mentions
bool attach(Desc &D, const Bound &b, bool eq, std::string &err)
{
    int v = -1;
    for (int u = 0; u < D.d; ++u) if (b.coef[u] != 0) v = u;
    if (v < 0) {
        if (eq ? b.c != 0 : b.c < 0) D.empty = true;
        return true;
    }
    const i64 c = b.coef[v];
    if (c != 1 && c != -1) { err = "coefficient of the last variable of a comparison must be 1 or -1"; return false; }
    Bound rest = b;
    rest.coef[v] = 0;
    // c = +1: x_v >= -rest ; c = -1: x_v <= rest
    Bound neg = rest;
    neg.c = -neg.c;
    for (int u = 0; u < MAXD; ++u) neg.coef[u] = -neg.coef[u];
    if (c == 1) { D.lo[v].push_back(neg); if (eq) D.hi[v].push_back(neg); }
    else { D.hi[v].push_back(rest); if (eq) D.lo[v].push_back(rest); }
    return true;
}

// Logical simplification of the bound lists: duplicates and bounds implied by a tighter one of the same form
// are dropped, constant bounds are folded into the dense extent (a constant lower bound raises `first`, a
// constant upper bound lowers `last`).
void simplify(Desc &D)
{
    for (int v = 0; v < D.d; ++v) {
        D.first[v] = 0;
        D.last[v] = D.dims[v] - 1;
        for (int side = 0; side < 2; ++side) {
            std::vector<Bound> &list = side ? D.hi[v] : D.lo[v];
            std::vector<Bound> keep;
            for (auto &b : list) {
                bool constant = true;
                for (int u = 0; u < MAXD; ++u) constant = constant && b.coef[u] == 0;
                if (constant) {
                    if (side) D.last[v] = std::min(D.last[v], b.c);
                    else D.first[v] = std::max(D.first[v], b.c);
                    continue;
                }
                // the same expression up to its constant: only the tighter bound is kept (x >= i - 2 and x >= i is
                // x >= i), which also drops exact duplicates
                bool dup = false;
                for (auto &k : keep)
                    if (std::equal(k.coef, k.coef + MAXD, b.coef)) {
                        k.c = side ? std::min(k.c, b.c) : std::max(k.c, b.c);
                        dup = true;
                    }
                if (!dup) keep.push_back(b);
            }
            list.swap(keep);
        }
        // a constant bound is implied when another bound stays on its safe side over the whole box of the
        // earlier variables (interval arithmetic on the affine expression)
        for (auto &b : D.lo[v]) {
            i64 mn = b.c;
            for (int u = 0; u < v; ++u) mn += b.coef[u] * (b.coef[u] > 0 ? D.first[u] : D.last[u]);
            if (mn >= D.first[v]) D.first_implied[v] = true;
        }
        for (auto &b : D.hi[v]) {
            i64 mx = b.c;
            for (int u = 0; u < v; ++u) mx += b.coef[u] * (b.coef[u] > 0 ? D.last[u] : D.first[u]);
            if (mx <= D.last[v]) D.last_implied[v] = true;
        }
    }
}

void range_of(const Desc &D, int v, const i64 *x, i64 &lo, i64 &hi)
{
    lo = D.first[v];
    hi = D.last[v];
    for (auto &b : D.lo[v]) lo = std::max(lo, bound_eval(b, x, v));
    for (auto &b : D.hi[v]) hi = std::min(hi, bound_eval(b, x, v));
}

void build_nest(Desc &D)
{
    std::string s;
    for (int v = 0; v < D.d; ++v) {
        std::vector<std::string> los, his;
        if (!D.first_implied[v]) los.push_back(std::to_string((long long)D.first[v]));
        if (!D.last_implied[v]) his.push_back(std::to_string((long long)D.last[v]));
        for (auto &b : D.lo[v]) los.push_back(bound_text(b, D.vars, v));
        for (auto &b : D.hi[v]) his.push_back(bound_text(b, D.vars, v));
        auto join = [](const std::vector<std::string> &a, const char *f) {
            if (a.size() == 1) return a[0];
            std::string r = std::string(f) + "(";
            for (size_t q = 0; q < a.size(); ++q) r += (q ? ", " : "") + a[q];
            return r + ")";
        };
        s += std::string(2 * v, ' ') + "for (" + D.vars[v] + " = " + join(los, "max") + "; " + D.vars[v] + " <= " +
             join(his, "min") + "; ++" + D.vars[v] + ")\n";
    }
    s += std::string(2 * D.d, ' ') + D.name + "_C[p++]\n";
    D.nest = s;
}

// start of the innermost run of every prefix (x_0 .. x_{d-2}), in nest order
bool build_tables(Desc &D, std::string &err)
{
    D.prefixes = 1;
    for (int v = 0; v + 1 < D.d; ++v) D.prefixes *= D.dims[v];
    i64 box = D.prefixes * D.dims[D.d - 1];
    if (D.prefixes > ((i64)1 << 26) || box > ((i64)1 << 31) - 1) { err = "index box too large"; return false; }
    D.table.assign((size_t)D.prefixes, -1);
    std::vector<int32_t> runs;
    i64 pos = 0;
    if (!D.empty) {
        i64 x[MAXD] = {0, 0, 0, 0};
        // iterative nest over the prefix variables
        const int np = D.d - 1;
        i64 lo[MAXD], hi[MAXD];
        int v = 0;
        bool done = false;
        if (np == 0) {
            i64 l, h;
            range_of(D, 0, x, l, h);
            if (l <= h) { D.table[0] = 0; runs.push_back(0); pos = h - l + 1; }
            done = true;
        } else {
            range_of(D, 0, x, lo[0], hi[0]);
            x[0] = lo[0];
        }
        while (!done) {
            if (x[v] > hi[v]) {
                if (v == 0) break;
                --v;
                ++x[v];
                continue;
            }
            if (v + 1 < np) {
                ++v;
                range_of(D, v, x, lo[v], hi[v]);
                x[v] = lo[v];
                continue;
            }
            // full prefix: innermost run
            i64 l, h;
            range_of(D, D.d - 1, x, l, h);
            if (l <= h) {
                i64 pf = 0;
                for (int u = 0; u < np; ++u) pf = pf * D.dims[u] + x[u];
                if (pos > ((i64)1 << 31) - 1 - (h - l + 1)) { err = "more than 2^31 unique entries"; return false; }
                D.table[(size_t)pf] = (int32_t)pos;
                runs.push_back((int32_t)pf);
                pos += h - l + 1;
            }
            ++x[v];
        }
    }
    D.count = pos;
    D.nruns = (i64)runs.size();
    D.table.insert(D.table.end(), runs.begin(), runs.end());
    // block tuples for the moment kernels: walk the runs and mark the blocks each one touches
    bool equal = D.d == 2 || D.d == 3;
    for (int v = 1; v < D.d; ++v) equal = equal && D.dims[v] == D.dims[0];
    if (equal && D.dims[0] <= 256) {
        const int d = D.d;
        D.mbs = d == 2 ? 8 : 4;                                  // 64 accumulators per lane either way
        const i64 nb = (D.dims[0] + D.mbs - 1) / D.mbs;
        D.mnp = nb * D.mbs;
        i64 nbt = 1;
        for (int v = 0; v < d; ++v) nbt *= nb;
        std::vector<char> mark((size_t)nbt, 0);
        for (i64 r = 0; r < D.nruns; ++r) {
            i64 pf = runs[(size_t)r], x[MAXD] = {0, 0, 0, 0};
            for (int v = d - 2; v >= 0; --v) { x[v] = pf % D.dims[v]; pf /= D.dims[v]; }
            i64 l, h;
            range_of(D, d - 1, x, l, h);
            i64 base = 0;
            for (int v = 0; v + 1 < d; ++v) base = base * nb + x[v] / D.mbs;
            for (i64 b = l / D.mbs; b <= h / D.mbs; ++b) mark[(size_t)(base * nb + b)] = 1;
        }
        for (i64 t = 0; t < nbt; ++t) {
            if (!mark[(size_t)t]) continue;
            i64 c[MAXD], q = t;
            for (int v = d - 1; v >= 0; --v) { c[v] = q % nb; q /= nb; }
            for (int v = 0; v < d; ++v) D.table.push_back((int32_t)c[v]);
            ++D.ntiles;
        }
    }
    return true;
}

std::string args_list(int n, const char *prefix, bool typed)
{
    std::string s;
    for (int u = 0; u < n; ++u) s += std::string(u ? ", " : "") + (typed ? "int " : "") + prefix + std::to_string(u);
    return s;
}

void build_source(Desc &D)
{
    const int d = D.d;
    std::string s;
    s += "// generated for " + D.name + ": unique set of order " + std::to_string(d) + "\n";
    s += "#define ST_D " + std::to_string(d) + "\n";
    s += "#define ST_PREFIXES " + std::to_string((long long)D.prefixes) + "\n";
    s += "#define ST_NRUNS " + std::to_string((long long)D.nruns) + "\n";
    s += "#define ST_COUNT " + std::to_string((long long)D.count) + "\n";
    for (int v = 0; v < d; ++v) s += "#define ST_DIM" + std::to_string(v) + " " + std::to_string((long long)D.dims[v]) + "\n";
    s += "static __device__ __forceinline__ int st_max(int a, int b) { return a > b ? a : b; }\n";
    s += "static __device__ __forceinline__ int st_min(int a, int b) { return a < b ? a : b; }\n";
    // bounds of every variable from the earlier ones: max of the lower bounds, min of the upper bounds
    for (int v = 0; v < d; ++v) {
        std::string a = args_list(v, "x", true);
        std::string lo = D.first_implied[v] ? "" : std::to_string((long long)D.first[v]);
        std::string hi = D.last_implied[v] ? "" : std::to_string((long long)D.last[v]);
        for (auto &b : D.lo[v]) lo = lo.empty() ? bound_code(b, v) : "st_max(" + lo + ", " + bound_code(b, v) + ")";
        for (auto &b : D.hi[v]) hi = hi.empty() ? bound_code(b, v) : "st_min(" + hi + ", " + bound_code(b, v) + ")";
        s += "static __device__ __forceinline__ int st_lo" + std::to_string(v) + "(" + a + ") { return " + lo + "; }\n";
        s += "static __device__ __forceinline__ int st_hi" + std::to_string(v) + "(" + a + ") { return " + hi + "; }\n";
    }
    // membership and packed position of an index tuple
    s += "static __device__ __forceinline__ bool st_in(" + args_list(d, "x", true) + ")\n{\n    return ";
    s += D.empty ? "false" : "true";
    for (int v = 0; v < d; ++v) {
        std::string a = args_list(v, "x", false), xv = "x" + std::to_string(v);
        s += "\n        && " + xv + " >= st_lo" + std::to_string(v) + "(" + a + ") && " + xv + " <= st_hi" + std::to_string(v) + "(" + a + ")";
    }
    s += ";\n}\n";
    std::string pf = "0";
    for (int v = 0; v + 1 < d; ++v) pf = "(" + pf + ") * ST_DIM" + std::to_string(v) + " + x" + std::to_string(v);
    s += "static __device__ __forceinline__ int st_rank(const int *tab, " + args_list(d, "x", true) + ")\n{\n";
    s += "    return tab[" + pf + "] + (x" + std::to_string(d - 1) + " - st_lo" + std::to_string(d - 1) + "(" + args_list(d - 1, "x", false) + "));\n}\n";
    // prefix id -> x0 .. x{d-2}
    s += "#define ST_DECODE_PREFIX(pf)";
    {
        std::string rem = "int st_r = (pf);";
        std::string body;
        for (int v = d - 2; v >= 0; --v) {
            body += " const int x" + std::to_string(v) + " = st_r % ST_DIM" + std::to_string(v) + "; st_r /= ST_DIM" + std::to_string(v) + ";";
        }
        s += " " + rem + body + " (void)st_r;\n";
    }
    const std::string pre = args_list(d - 1, "x", false);
    const std::string last = "x" + std::to_string(d - 1);
    std::string dense = "0";
    for (int v = 0; v < d; ++v) dense = "((long long)(" + dense + ")) * ST_DIM" + std::to_string(v) + " + x" + std::to_string(v);
    // list: one wave per run, lanes along the last variable
    s += "extern \"C\" __global__ void st_gen_list(const int *__restrict__ tab, int *__restrict__ out)\n{\n";
    s += "    const int run = blockIdx.x * (blockDim.x / 64) + threadIdx.x / 64, lane = threadIdx.x % 64;\n";
    s += "    if (run >= ST_NRUNS) return;\n    const int pf = tab[ST_PREFIXES + run];\n    ST_DECODE_PREFIX(pf)\n";
    s += "    const int lo = st_lo" + std::to_string(d - 1) + "(" + pre + "), hi = st_hi" + std::to_string(d - 1) + "(" + pre + "), start = tab[pf];\n";
    s += "    for (int " + last + " = lo + lane; " + last + " <= hi; " + last + " += 64) {\n";
    s += "        int *o = out + (long long)(start + " + last + " - lo) * ST_D;\n";
    for (int v = 0; v < d; ++v) s += "        o[" + std::to_string(v) + "] = x" + std::to_string(v) + ";\n";
    s += "    }\n}\n";
    // thp: Ac(p) = Bc(p) * C(x(p)), C dense
    s += "extern \"C\" __global__ void st_gen_thp(const int *__restrict__ tab, const float *__restrict__ Bc,\n"
         "                                      const float *__restrict__ C, float *__restrict__ Ac)\n{\n";
    s += "    const int run = blockIdx.x * (blockDim.x / 64) + threadIdx.x / 64, lane = threadIdx.x % 64;\n";
    s += "    if (run >= ST_NRUNS) return;\n    const int pf = tab[ST_PREFIXES + run];\n    ST_DECODE_PREFIX(pf)\n";
    s += "    const int lo = st_lo" + std::to_string(d - 1) + "(" + pre + "), hi = st_hi" + std::to_string(d - 1) + "(" + pre + "), start = tab[pf];\n";
    s += "    for (int " + last + " = lo + lane; " + last + " <= hi; " + last + " += 64) {\n";
    s += "        const int p = start + " + last + " - lo;\n";
    s += "        Ac[p] = Bc[p] * C[" + dense + "];\n    }\n}\n";
    // value of one dense element: Tc(rank(x)) on the unique set, Tc(rank(x')) through the redundancy map, 0 elsewhere
    const std::string xs = args_list(d, "x", false);
    s += "static __device__ __forceinline__ int st_pos(const int *__restrict__ tab, " + args_list(d, "x", true) + ")\n{\n";
    s += "    int pos = -1;\n";
    s += "    if (st_in(" + xs + ")) pos = st_rank(tab, " + xs + ");\n";
    if (D.red_sort) {
        s += "    else {\n        int y[ST_D] = {" + xs + "};\n";
        s += "        for (int a = 1; a < ST_D; ++a)\n            for (int b = a; b > 0 && y[b - 1] > y[b]; --b) { const int t = y[b]; y[b] = y[b - 1]; y[b - 1] = t; }\n";
        std::string ys;
        for (int v = 0; v < d; ++v) ys += std::string(v ? ", " : "") + "y[" + std::to_string(v) + "]";
        s += "        if (st_in(" + ys + ")) pos = st_rank(tab, " + ys + ");\n    }\n";
    }
    for (auto &t : D.red) {
        s += "    if (pos < 0";
        for (auto &c : t.cond) s += " && " + bound_code(c, d) + " >= 0";
        s += ") {\n";
        std::string ys;
        for (int v = 0; v < d; ++v) {
            s += "        const int y" + std::to_string(v) + " = " + bound_code(t.map[v], d) + ";\n";
            ys += std::string(v ? ", " : "") + "y" + std::to_string(v);
        }
        s += "        if (st_in(" + ys + ")) pos = st_rank(tab, " + ys + ");\n    }\n";
    }
    s += "    return pos;\n}\n";
    s += "static __device__ __forceinline__ float st_value(const int *__restrict__ tab, const float *__restrict__ Tc, " +
         args_list(d, "x", true) + ")\n{\n";
    s += "    const int pos = st_pos(tab, " + xs + ");\n    return pos >= 0 ? Tc[pos] : 0.f;\n}\n";
    // expand: one thread per dense element, or per four consecutive ones along the last variable (one 16-byte store)
    const bool vec = D.dims[d - 1] % 4 == 0;
    const std::string lastdim = "ST_DIM" + std::to_string(d - 1);
    s += "extern \"C\" __global__ void st_gen_expand(const int *__restrict__ tab, const float *__restrict__ Tc,\n"
         "                                         float *__restrict__ T)\n{\n";
    std::string total = "1LL";
    for (int v = 0; v < d; ++v) total += " * ST_DIM" + std::to_string(v);
    s += "    const long long e = (long long)blockIdx.x * blockDim.x + threadIdx.x;\n";
    s += "    if (e >= " + total + (vec ? " / 4" : "") + ") return;\n";
    s += "    long long st_r = e;\n";
    for (int v = d - 1; v >= 0; --v) {
        const std::string dim = "ST_DIM" + std::to_string(v);
        if (v == d - 1 && vec)
            s += "    const int x" + std::to_string(v) + " = 4 * (int)(st_r % (" + dim + " / 4)); st_r /= " + dim + " / 4;\n";
        else
            s += "    const int x" + std::to_string(v) + " = (int)(st_r % " + dim + "); st_r /= " + dim + ";\n";
    }
    if (vec) {
        const std::string pre2 = d > 1 ? args_list(d - 1, "x", false) + ", " : std::string();
        const std::string xl = "x" + std::to_string(d - 1);
        s += "    float4 v;\n";
        const char *comp[4] = {"x", "y", "z", "w"};
        for (int q = 0; q < 4; ++q)
            s += std::string("    v.") + comp[q] + " = st_value(tab, Tc, " + pre2 + xl + " + " + std::to_string(q) + ");\n";
        s += "    *reinterpret_cast<float4 *>(T + 4 * e) = v;\n}\n";
    } else {
        s += "    T[e] = st_value(tab, Tc, " + xs + ");\n}\n";
    }
    // expand onto: the same reconstruction, but only the elements this structure holds (stored, or reached through
    // its redundancy map) are written; everything else keeps what the dense array held -- the second and later
    // summands of a structure that is a sum of nests (the direct sum) are laid over the first this way
    s += "extern \"C\" __global__ void st_gen_expand_onto(const int *__restrict__ tab, const float *__restrict__ Tc,\n"
         "                                              float *__restrict__ T)\n{\n";
    s += "    const long long e = (long long)blockIdx.x * blockDim.x + threadIdx.x;\n";
    s += "    if (e >= " + total + ") return;\n";
    s += "    long long st_r = e;\n";
    for (int v = d - 1; v >= 0; --v) {
        const std::string dim = "ST_DIM" + std::to_string(v);
        s += "    const int x" + std::to_string(v) + " = (int)(st_r % " + dim + "); st_r /= " + dim + ";\n";
    }
    s += "    const int pos = st_pos(tab, " + xs + ");\n    if (pos >= 0) T[e] = Tc[pos];\n}\n";
    // gather: the value of the structured tensor at a LIST of dense positions (unique set, redundancy map or
    // zero, as in the reconstruction), optionally times a factor per position -- what an element-wise product
    // with another structured operand needs, evaluated only where the product's unique set says
    s += "extern \"C\" __global__ void st_gen_gather(const int *__restrict__ tab, const float *__restrict__ Tc,\n"
         "                                         const int *__restrict__ idx, long long count, int stride, int offset,\n"
         "                                         const float *__restrict__ scale, const float *__restrict__ addend,\n"
         "                                         float *__restrict__ out)\n{\n";
    s += "    const long long p = (long long)blockIdx.x * blockDim.x + threadIdx.x;\n    if (p >= count) return;\n";
    {
        std::string at;
        for (int v = 0; v < d; ++v) {
            const std::string xv = "x" + std::to_string(v);
            s += "    const int " + xv + " = idx[p * stride + offset + " + std::to_string(v) + "];\n";
            at += std::string(v ? " && " : "") + xv + " >= 0 && " + xv + " < ST_DIM" + std::to_string(v);
        }
        s += "    const float v = (" + at + ") ? st_value(tab, Tc, " + xs + ") : 0.f;\n";
    }
    s += "    const float w = scale ? scale[p] * v : v;\n    out[p] = addend ? w + addend[p] : w;\n}\n";
    // marginalization of the last variable: out(run) = sum of the entries of the run, in a fixed order (the lanes'
    // partial sums in lane order); a group of L = min(64, workgroup size) threads per run
    s += "extern \"C\" __global__ void st_gen_sum_last(const int *__restrict__ tab, const float *__restrict__ Bc,\n"
         "                                           float *__restrict__ out)\n{\n";
    s += "    __shared__ float st_lane[256];\n";
    s += "    const int tid = threadIdx.x, nt = blockDim.x, L = nt < 64 ? nt : 64, ln = tid % L, g = tid / L;\n";
    s += "    const int run = blockIdx.x * (nt / L) + g;\n";
    s += "    float acc = 0.f;\n";
    s += "    int start = 0;\n";
    s += "    if (run < ST_NRUNS) {\n        const int pf = tab[ST_PREFIXES + run];\n        ST_DECODE_PREFIX(pf)\n";
    s += "        const int lo = st_lo" + std::to_string(d - 1) + "(" + pre + "), hi = st_hi" + std::to_string(d - 1) + "(" + pre + ");\n";
    s += "        start = tab[pf];\n";
    s += "        for (int p = ln; p <= hi - lo; p += L) acc += Bc[start + p];\n    }\n";
    s += "    st_lane[tid] = acc;\n    __syncthreads();\n";
    s += "    if (ln == 0 && run < ST_NRUNS) {\n        float v = 0.f;\n        for (int q = 0; q < L; ++q) v += st_lane[g * L + q];\n";
    s += "        out[run] = v;\n    }\n}\n";
    if (d == 3) {
        // MTTKRP of the kernel table over the unique set: A(x0, r) = sum over the stored (x1, x2) of row x0 of
        // Bc(rank(x)) * C(x1, r) * D(x2, r).  One workgroup per output row x0 and block of 16 columns r; its
        // waves take the runs (x1) of the row in turn, the lanes the entries of a run; sixteen accumulators per
        // thread, added over the threads in two levels, each in a fixed order.  Written so that a
        // launch with any number of threads per workgroup (also one) computes the same sums.
        s += "#define ST_MK_COLS 16\n#define ST_MK_MAXT 1024\n#define ST_MK_PARTS 16\n";
        // sixteen consecutive values of a row of C or D (zeros past the last column); 16-byte loads when the rows
        // are 16-byte aligned (R a multiple of 4)
        s += "static __device__ __forceinline__ void st_mk_row(float (&o)[ST_MK_COLS], const float *__restrict__ p, int left, bool v4)\n{\n";
        s += "    if (v4) {\n        for (int q = 0; q < ST_MK_COLS / 4; ++q) {\n";
        s += "            float4 t = make_float4(0.f, 0.f, 0.f, 0.f);\n";
        s += "            if (4 * q < left) t = *reinterpret_cast<const float4 *>(p + 4 * q);\n";
        s += "            o[4 * q] = t.x; o[4 * q + 1] = t.y; o[4 * q + 2] = t.z; o[4 * q + 3] = t.w;\n        }\n";
        s += "    } else {\n        for (int c = 0; c < ST_MK_COLS; ++c) o[c] = c < left ? p[c] : 0.f;\n    }\n}\n";
        s += "extern \"C\" __global__ void st_gen_mttkrp(const int *__restrict__ tab, const float *__restrict__ Bc,\n"
             "                                         const float *__restrict__ C, const float *__restrict__ Dm,\n"
             "                                         float *__restrict__ A, int R)\n{\n";
        s += "    __shared__ float st_red[ST_MK_COLS][ST_MK_MAXT];\n";
        s += "    __shared__ float st_red2[ST_MK_COLS][ST_MK_PARTS];\n";
        s += "    const int tid = threadIdx.x, nt = blockDim.x, L = nt < 64 ? nt : 64, ln = tid % L, wv = tid / L, nw = nt / L;\n";
        s += "    const int x0 = blockIdx.x, r0 = blockIdx.y * ST_MK_COLS;\n";
        s += "    const bool v4 = (R & 3) == 0;\n";
        s += "    float acc[ST_MK_COLS];\n    for (int c = 0; c < ST_MK_COLS; ++c) acc[c] = 0.f;\n";
        s += "    if (ST_COUNT > 0 && x0 >= st_lo0() && x0 <= st_hi0()) {      // (an empty unique set: zeros)\n";
        s += "        for (int x1 = st_lo1(x0) + wv; x1 <= st_hi1(x0); x1 += nw) {\n";
        s += "            const int lo = st_lo2(x0, x1), hi = st_hi2(x0, x1);\n";
        s += "            if (lo > hi) continue;\n";
        s += "            const int start = tab[x0 * ST_DIM1 + x1];\n";
        s += "            float cr[ST_MK_COLS];\n";
        s += "            st_mk_row(cr, C + (long long)x1 * R + r0, R - r0, v4);\n";
        s += "#pragma unroll 2\n";
        s += "            for (int x2 = lo + ln; x2 <= hi; x2 += L) {\n";
        s += "                const float b = Bc[start + x2 - lo];\n";
        s += "                float dr[ST_MK_COLS];\n";
        s += "                st_mk_row(dr, Dm + (long long)x2 * R + r0, R - r0, v4);\n";
        s += "                for (int c = 0; c < ST_MK_COLS; ++c) acc[c] += (b * cr[c]) * dr[c];\n";
        s += "            }\n        }\n    }\n";
        s += "    for (int c = 0; c < ST_MK_COLS; ++c) st_red[c][tid] = acc[c];\n";
        s += "    __syncthreads();\n";
        // two levels, both in a fixed order: sixteen parts of consecutive threads per column, then the parts
        s += "    const int per = (nt + ST_MK_PARTS - 1) / ST_MK_PARTS;\n";
        s += "    for (int q = tid; q < ST_MK_COLS * ST_MK_PARTS; q += nt) {\n";
        s += "        const int c = q / ST_MK_PARTS, part = q % ST_MK_PARTS;\n";
        s += "        float v = 0.f;\n";
        s += "        for (int t = part * per; t < (part + 1) * per && t < nt; ++t) v += st_red[c][t];\n";
        s += "        st_red2[c][part] = v;\n    }\n";
        s += "    __syncthreads();\n";
        s += "    for (int c = tid; c < ST_MK_COLS && r0 + c < R; c += nt) {\n";
        s += "        float v = 0.f;\n        for (int part = 0; part < ST_MK_PARTS; ++part) v += st_red2[c][part];\n";
        s += "        A[(long long)x0 * R + r0 + c] = v;\n    }\n}\n";
        // second half of the matrix-core route (last variable free: every run is a whole fibre): Y(run, r) =
        // sum_l Bc(run, l) D(l, r) comes from the TTM kernels; here A(x0, r) = sum over the runs (x0, x1) of
        // C(x1, r) * Y(run, r).  A workgroup per row x0 and block of 64 columns; the runs of a row are consecutive
        // in the run list (first one by binary search), dealt to ST_MC_SLOTS thread groups, partial sums added in
        // slot order.
        s += "#define ST_MC_SLOTS 16\n";
        s += "extern \"C\" __global__ void st_gen_mttkrp_combine(const int *__restrict__ tab, const float *__restrict__ Y,\n"
             "                                                 const float *__restrict__ C, float *__restrict__ A, int R)\n{\n";
        s += "    __shared__ float st_part[ST_MC_SLOTS][64];\n";
        s += "    const int tid = threadIdx.x, nt = blockDim.x, L = nt < 64 ? nt : 64, ln = tid % L, sl = tid / L, ns = nt / L;\n";
        s += "    const int x0 = blockIdx.x, r0 = blockIdx.y * 64;\n";
        s += "    const int *runs = tab + ST_PREFIXES;\n";
        s += "    int ra = 0, re = ST_NRUNS;                       // first run whose prefix belongs to row x0 or a later one\n";
        s += "    while (ra < re) { const int mid = (ra + re) / 2; if (runs[mid] / ST_DIM1 < x0) ra = mid + 1; else re = mid; }\n";
        s += "    int rb = ra;                                     // ... to row x0 + 1 or a later one\n";
        s += "    re = ST_NRUNS;\n";
        s += "    while (rb < re) { const int mid = (rb + re) / 2; if (runs[mid] / ST_DIM1 <= x0) rb = mid + 1; else re = mid; }\n";
        s += "    for (int cb = 0; cb < 64; cb += L) {              // (one pass when the workgroup has 64 lanes per slot)\n";
        s += "        const int r = r0 + cb + ln;\n";
        s += "        float acc = 0.f;\n";
        s += "        if (r < R) {\n";
        s += "#pragma unroll 4\n";
        s += "            for (int run = ra + sl; run < rb; run += ns)\n";
        s += "                acc += C[(long long)(runs[run] % ST_DIM1) * R + r] * Y[(long long)run * R + r];\n";
        s += "        }\n";
        s += "        st_part[sl][ln] = acc;\n";
        s += "        __syncthreads();\n";
        s += "        if (sl == 0 && r < R) {\n";
        s += "            float v = 0.f;\n            for (int q = 0; q < ns; ++q) v += st_part[q][ln];\n";
        s += "            A[(long long)x0 * R + r] = v;\n        }\n";
        s += "        __syncthreads();\n    }\n}\n";
    }
    if (D.ntiles > 0) {
        // moment accumulation over the unique set: Sc(rank(x)) (+)= sum_s prod_v X(s, x_v).  One lane per block
        // tuple with its ST_MBS^d = 64 accumulators in registers, sample rows staged through a double-buffered
        // LDS chunk, sample slices over grid.y; a second kernel adds the slice partials in a fixed order, keeps
        // the tuples of the unique set and scatters them through st_rank.
        const int bs = (int)D.mbs;
        s += "#define ST_MBS " + std::to_string(bs) + "\n#define ST_NTILES " + std::to_string((long long)D.ntiles) +
             "\n#define ST_MNP " + std::to_string((long long)D.mnp) + "\n#define ST_TILES_OFF (ST_PREFIXES + ST_NRUNS)\n"
             "#ifndef ST_DYN_LDS\n#define ST_DYN_LDS extern __shared__ float st_gen_lds[];\n#endif\n";
        s += "extern \"C\" __global__ void st_gen_moment(const int *__restrict__ tab, const float *__restrict__ X, long long N,\n"
             "                                         int ch, long long slice, float *__restrict__ ws)\n{\n";
        s += "    ST_DYN_LDS\n";
        s += "    const int tid = threadIdx.x, nthreads = blockDim.x, np4 = ST_MNP / 4, pieces = ch * np4, chunk_f = ch * ST_MNP;\n";
        s += "    const int t = blockIdx.x * nthreads + tid, tc = t < ST_NTILES ? t : ST_NTILES - 1;\n";
        for (int v = 0; v < d; ++v)
            s += "    const int o" + std::to_string(v) + " = ST_MBS * tab[ST_TILES_OFF + tc * ST_D + " + std::to_string(v) + "];\n";
        s += "    const long long s_begin = (long long)blockIdx.y * slice, s_end = s_begin + slice < N ? s_begin + slice : N;\n";
        s += "    const long long nchunks = s_end > s_begin ? (s_end - s_begin + ch - 1) / ch : 0;\n";
        s += "    float acc[64];\n    for (int e = 0; e < 64; ++e) acc[e] = 0.f;\n";
        s += "    for (long long c = 0; c < nchunks; ++c) {\n";
        s += "        const long long s0 = s_begin + c * ch;\n";
        s += "        float *buf = st_gen_lds + (int)(c & 1) * chunk_f;          // double buffered: one barrier per chunk\n";
        s += "        for (int j = tid; j < pieces; j += nthreads) {\n";
        s += "            const int smp = j / np4, c0 = 4 * (j - smp * np4);\n";
        s += "            const long long sq = s0 + smp, sc = sq < s_end ? sq : s_end - 1;\n";
        s += "            const float *row = X + sc * ST_DIM0;\n";
        s += "            float4 v;\n";
        if (D.dims[0] % 4 == 0) {       // rows are 16-byte aligned and have no ragged end
            s += "            v = *reinterpret_cast<const float4 *>(row + c0);\n";
            s += "            if (sq >= s_end) v = make_float4(0.f, 0.f, 0.f, 0.f);\n";
        } else {
        s += "            v.x = (sq < s_end && c0 + 0 < ST_DIM0) ? row[c0 + 0 < ST_DIM0 ? c0 + 0 : ST_DIM0 - 1] : 0.f;\n";
        s += "            v.y = (sq < s_end && c0 + 1 < ST_DIM0) ? row[c0 + 1 < ST_DIM0 ? c0 + 1 : ST_DIM0 - 1] : 0.f;\n";
        s += "            v.z = (sq < s_end && c0 + 2 < ST_DIM0) ? row[c0 + 2 < ST_DIM0 ? c0 + 2 : ST_DIM0 - 1] : 0.f;\n";
        s += "            v.w = (sq < s_end && c0 + 3 < ST_DIM0) ? row[c0 + 3 < ST_DIM0 ? c0 + 3 : ST_DIM0 - 1] : 0.f;\n";
        }
        s += "            *reinterpret_cast<float4 *>(buf + 4 * j) = v;\n        }\n";
        s += "        __syncthreads();\n";
        s += "        const float *row = buf;\n";
        s += "        for (int smp = 0; smp < ch; ++smp, row += ST_MNP) {\n";
        if (d == 3) {
            s += "            const float4 a = *reinterpret_cast<const float4 *>(row + o0), b = *reinterpret_cast<const float4 *>(row + o1), cc = *reinterpret_cast<const float4 *>(row + o2);\n";
            s += "            const float xa[4] = {a.x, a.y, a.z, a.w}, xb[4] = {b.x, b.y, b.z, b.w}, xc[4] = {cc.x, cc.y, cc.z, cc.w};\n";
            s += "#pragma unroll\n            for (int i = 0; i < 4; ++i)\n#pragma unroll\n                for (int j = 0; j < 4; ++j) {\n                    const float p = xa[i] * xb[j];\n#pragma unroll\n                    for (int k = 0; k < 4; ++k) acc[(i * 4 + j) * 4 + k] += p * xc[k];\n                }\n";
        } else {
            s += "            const float4 a0 = *reinterpret_cast<const float4 *>(row + o0), a1 = *reinterpret_cast<const float4 *>(row + o0 + 4);\n";
            s += "            const float4 b0 = *reinterpret_cast<const float4 *>(row + o1), b1 = *reinterpret_cast<const float4 *>(row + o1 + 4);\n";
            s += "            const float xa[8] = {a0.x, a0.y, a0.z, a0.w, a1.x, a1.y, a1.z, a1.w}, xb[8] = {b0.x, b0.y, b0.z, b0.w, b1.x, b1.y, b1.z, b1.w};\n";
            s += "#pragma unroll\n            for (int i = 0; i < 8; ++i)\n#pragma unroll\n                for (int j = 0; j < 8; ++j) acc[i * 8 + j] += xa[i] * xb[j];\n";
        }
        s += "        }\n    }\n";
        s += "    if (t < ST_NTILES) {\n        float *dst = ws + ((long long)blockIdx.y * ST_NTILES + t) * 64;\n";
        s += "        for (int e = 0; e < 64; ++e) dst[e] = acc[e];\n    }\n}\n";
        // reduce: 16 accumulators x 16 slice groups per block
        s += "extern \"C\" __global__ void st_gen_moment_reduce(const int *__restrict__ tab, const float *__restrict__ ws, int S,\n"
             "                                                float *__restrict__ Sc, int accumulate)\n{\n";
        s += "    __shared__ float part[16][16];\n";
        s += "    const int a = threadIdx.x & 15, g = threadIdx.x >> 4;\n    const long long t = (long long)blockIdx.x * 16 + a;\n";
        s += "    float sum = 0.f;\n    if (t < (long long)ST_NTILES * 64)\n        for (int y = g; y < S; y += 16) sum += ws[(long long)y * ST_NTILES * 64 + t];\n";
        s += "    part[g][a] = sum;\n    __syncthreads();\n    if (g != 0 || t >= (long long)ST_NTILES * 64) return;\n";
        s += "    float v = 0.f;\n    for (int q = 0; q < 16; ++q) v += part[q][a];\n";
        s += "    const int tile = (int)(t >> 6), e = (int)(t & 63);\n";
        if (d == 3) {
            s += "    const int x0 = ST_MBS * tab[ST_TILES_OFF + tile * 3] + (e >> 4), x1 = ST_MBS * tab[ST_TILES_OFF + tile * 3 + 1] + ((e >> 2) & 3),\n"
                 "              x2 = ST_MBS * tab[ST_TILES_OFF + tile * 3 + 2] + (e & 3);\n";
        } else {
            s += "    const int x0 = ST_MBS * tab[ST_TILES_OFF + tile * 2] + (e >> 3), x1 = ST_MBS * tab[ST_TILES_OFF + tile * 2 + 1] + (e & 7);\n";
        }
        s += "    if (!st_in(" + xs + ")) return;\n";
        s += "    const int p = st_rank(tab, " + xs + ");\n    Sc[p] = accumulate ? Sc[p] + v : v;\n}\n";
    }
    D.source = s;
}

// Property 1 of the semantics (T_U * T_R is empty): no index may be both a stored entry and the source of a
// redundancy term.  Every run of the unique set (prefix fixed, last variable in [l, h]) is cut against the
// term's condition, which for a fixed prefix is an interval of the last variable.
bool first_overlap(const Desc &D, size_t term, i64 *where)
{
    const RedTerm &t = D.red[term];
    const int d = D.d, np = d - 1;
    for (i64 r = 0; r < D.nruns; ++r) {
        i64 pf = D.table[(size_t)(D.prefixes + r)], x[MAXD] = {0, 0, 0, 0};
        for (int v = np - 1; v >= 0; --v) { x[v] = pf % D.dims[v]; pf /= D.dims[v]; }
        i64 l, h;
        range_of(D, np, x, l, h);
        bool none = false;
        for (auto &c : t.cond) {                       // c.c + sum coef*x >= 0
            i64 rest = c.c;
            for (int u = 0; u < np; ++u) rest += c.coef[u] * x[u];
            const i64 a = c.coef[np];
            if (a == 0) { if (rest < 0) none = true; }
            else if (a > 0) l = std::max(l, -(rest >= 0 ? rest / a : -((-rest + a - 1) / a)));      // x >= ceil(-rest / a)
            else h = std::min(h, rest >= 0 ? rest / (-a) : -((-rest + (-a) - 1) / (-a)));           // x <= floor(rest / -a)
            if (none) break;
        }
        if (!none && l <= h) {
            for (int u = 0; u < np; ++u) where[u] = x[u];
            where[np] = l;
            return true;
        }
    }
    return false;
}

// simplification, nest, tables, Property 1, generated source: the common tail of every way to make a descriptor
st_status finish(Desc &D)
{
    simplify(D);
    build_nest(D);
    if (!build_tables(D, D.error)) return ST_ERR_UNSUPPORTED;
    for (size_t q = 0; q < D.red.size(); ++q) {
        i64 at[MAXD];
        if (first_overlap(D, q, at)) {
            D.error = "redundancy term " + std::to_string(q + 1) + " applies to the stored entry (";
            for (int v = 0; v < D.d; ++v) D.error += (v ? "," : "") + std::to_string((long long)at[v]);
            D.error += "): the unique set and the redundancy map must be disjoint (T_U * T_R is empty)";
            return ST_ERR_SHAPE;
        }
    }
    build_source(D);
    return ST_OK;
}

st_status parse_all(Desc &D, const char *unique_set, const char *redundancy, const i64 *dims, int ndims,
                    const char *const *pnames, const i64 *pvalues, int nparams)
{
    std::map<std::string, i64> params;
    for (int q = 0; q < nparams; ++q) {
        if (!pnames[q]) { D.error = "NULL parameter name"; return ST_ERR_NULL; }
        params[pnames[q]] = pvalues[q];
    }
    Parser ps(unique_set);
    D.name = ps.ident();
    if (D.name.empty() || !ps.eat('(')) { D.error = "expected NAME(vars): factors"; return ST_ERR_SHAPE; }
    do {
        std::string v = ps.ident();
        if (v.empty()) { D.error = "expected an index variable"; return ST_ERR_SHAPE; }
        if (std::find(D.vars.begin(), D.vars.end(), v) != D.vars.end() || params.count(v)) {
            D.error = "name '" + v + "' used twice";
            return ST_ERR_SHAPE;
        }
        D.vars.push_back(v);
    } while (ps.eat(','));
    if (!ps.eat(')') || !ps.eat(':')) { D.error = "expected NAME(vars): factors"; return ST_ERR_SHAPE; }
    D.d = (int)D.vars.size();
    if (D.d < 1 || D.d > MAXD) { D.error = "order must be 1..4"; return ST_ERR_UNSUPPORTED; }
    if (D.d != ndims) { D.error = "number of sizes differs from the number of index variables"; return ST_ERR_SHAPE; }
    for (int v = 0; v < D.d; ++v) {
        if (dims[v] < 1 || dims[v] > ((i64)1 << 24)) { D.error = "size out of range"; return ST_ERR_SHAPE; }
        D.dims[v] = dims[v];
    }
    std::vector<Constraint> cons;
    if (!parse_product(ps, cons) || !ps.ok) { D.error = "cannot parse the unique set"; return ST_ERR_SHAPE; }
    ps.ws();
    if (*ps.p) { D.error = std::string("trailing text in the unique set: '") + ps.p + "'"; return ST_ERR_SHAPE; }
    for (auto &c : cons) {
        Bound b;
        if (!to_bound(c.e, D, params, b, D.error)) return ST_ERR_SHAPE;
        if (!attach(D, b, c.eq, D.error)) return ST_ERR_UNSUPPORTED;
    }
    if (redundancy && *redundancy) {
        Parser pr(redundancy);
        pr.ws();
        if (strncmp(pr.p, "sort", 4) == 0) {
            pr.p += 4;
            pr.ws();
            if (*pr.p) { D.error = "trailing text after 'sort'"; return ST_ERR_SHAPE; }
            D.red_sort = true;
            for (int v = 1; v < D.d; ++v)
                if (D.dims[v] != D.dims[0]) { D.error = "'sort' needs equal sizes"; return ST_ERR_SHAPE; }
        } else {
            do {
                std::vector<Constraint> cc;
                if (!parse_product(pr, cc)) { D.error = "cannot parse a redundancy condition"; return ST_ERR_SHAPE; }
                pr.ws();
                if (!(pr.p[0] == '-' && pr.p[1] == '>')) { D.error = "expected '->' in a redundancy term"; return ST_ERR_SHAPE; }
                pr.p += 2;
                if (!pr.eat('(')) { D.error = "expected '(' after '->'"; return ST_ERR_SHAPE; }
                RedTerm t;
                for (auto &c : cc) {
                    Bound b;
                    if (!to_bound(c.e, D, params, b, D.error)) return ST_ERR_SHAPE;
                    t.cond.push_back(b);
                    if (c.eq) {               // E == 0  <=>  E >= 0 and -E >= 0
                        Bound nb = b;
                        nb.c = -nb.c;
                        for (int u = 0; u < MAXD; ++u) nb.coef[u] = -nb.coef[u];
                        t.cond.push_back(nb);
                    }
                }
                for (int v = 0; v < D.d; ++v) {
                    Affine e;
                    if (!pr.expr(e)) { D.error = "cannot parse a redundancy target"; return ST_ERR_SHAPE; }
                    if (!to_bound(e, D, params, t.map[v], D.error)) return ST_ERR_SHAPE;
                    if (v + 1 < D.d && !pr.eat(',')) { D.error = "a redundancy target needs one expression per index"; return ST_ERR_SHAPE; }
                }
                if (!pr.eat(')')) { D.error = "expected ')' after a redundancy target"; return ST_ERR_SHAPE; }
                D.red.push_back(t);
            } while (pr.eat(';'));
            pr.ws();
            if (*pr.p || !pr.ok) { D.error = "trailing text in the redundancy map"; return ST_ERR_SHAPE; }
        }
    }
    return finish(D);
}

// ---- structure inference for an element-wise product ------------------------------------------------
// A(x) := M(x) * V(x) over the same index vector.  General rule of the inference figure:
//     A_U = M_U * V_U  +  M_U * V_R  +  M_R * V_U,        A_R = M_R * V_R,
// every summand a product of comparisons.  Simplification: a product whose comparisons contradict each other
// is the empty set and drops out of the sum (decided here by deriving its nest and counting: zero entries).
// What remains must be ONE product (a descriptor holds one); in A_R a pair of terms survives when both send x
// to the same unique index.
void add_box(Desc &D, const Desc &S)          // the comparisons of a finished descriptor: ranges and bound lists
{
    for (int v = 0; v < S.d; ++v) {
        Bound b;
        for (int u = 0; u < MAXD; ++u) b.coef[u] = 0;
        b.c = S.first[v];
        D.lo[v].push_back(b);
        b.c = S.last[v];
        D.hi[v].push_back(b);
        for (auto &q : S.lo[v]) D.lo[v].push_back(q);
        for (auto &q : S.hi[v]) D.hi[v].push_back(q);
    }
    D.empty = D.empty || S.empty;
}

std::vector<RedTerm> terms_of(const Desc &S)   // 'sort' of order 2 is the class-S map (x1 < x0) -> (x1, x0)
{
    std::vector<RedTerm> out = S.red;
    if (S.red_sort && S.d == 2) {
        RedTerm t;
        Bound c;
        for (int u = 0; u < MAXD; ++u) c.coef[u] = 0;
        c.c = -1; c.coef[0] = 1; c.coef[1] = -1;                 // x0 - x1 - 1 >= 0
        t.cond.push_back(c);
        for (int v = 0; v < MAXD; ++v) { t.map[v].c = 0; for (int u = 0; u < MAXD; ++u) t.map[v].coef[u] = 0; }
        t.map[0].coef[1] = 1;
        t.map[1].coef[0] = 1;
        out.push_back(t);
    }
    return out;
}

bool same_map(const RedTerm &a, const RedTerm &b, int d)
{
    for (int v = 0; v < d; ++v)
        if (a.map[v].c != b.map[v].c || !std::equal(a.map[v].coef, a.map[v].coef + MAXD, b.map[v].coef)) return false;
    return true;
}

st_status infer_product(const Desc &M, const Desc &V, Desc &A)
{
    if (M.d != V.d || !std::equal(M.dims, M.dims + MAXD, V.dims)) { A.error = "operands of different shape"; return ST_ERR_SHAPE; }
    if ((M.red_sort || V.red_sort) && M.d != 2) {
        A.error = "a 'sort' redundancy map of order above 2 is a sum of conditions: not supported in a product";
        return ST_ERR_UNSUPPORTED;
    }
    const int d = M.d;
    const std::vector<RedTerm> mr = terms_of(M), vr = terms_of(V);
    // the summands of A_U, each as a candidate descriptor; kept when not empty
    struct Cand { const Desc *u; const RedTerm *t; const Desc *other; };
    std::vector<Cand> cands;
    cands.push_back(Cand{&M, nullptr, &V});
    for (auto &t : vr) cands.push_back(Cand{&M, &t, nullptr});
    for (auto &t : mr) cands.push_back(Cand{&V, &t, nullptr});
    int kept = -1, nkept = 0;
    for (size_t q = 0; q < cands.size(); ++q) {
        Desc T;
        T.d = d; T.name = "A"; T.vars = M.vars;
        std::copy(M.dims, M.dims + MAXD, T.dims);
        add_box(T, *cands[q].u);
        if (cands[q].other) add_box(T, *cands[q].other);
        std::string err;
        bool ok = true;
        if (cands[q].t) for (auto &c : cands[q].t->cond) ok = ok && attach(T, c, false, err);
        if (!ok) { A.error = "a redundancy condition cannot be turned into loop bounds: " + err; return ST_ERR_UNSUPPORTED; }
        simplify(T);
        if (!build_tables(T, err)) { A.error = err; return ST_ERR_UNSUPPORTED; }
        if (T.count > 0) { kept = (int)q; ++nkept; }
    }
    A.d = d; A.name = "A"; A.vars = M.vars;
    std::copy(M.dims, M.dims + MAXD, A.dims);
    if (nkept > 1) {
        A.error = "the unique set of the product is a sum of " + std::to_string(nkept) + " non-empty products; a descriptor holds one";
        return ST_ERR_UNSUPPORTED;
    }
    if (nkept == 0) A.empty = true;
    else {
        add_box(A, *cands[(size_t)kept].u);
        if (cands[(size_t)kept].other) add_box(A, *cands[(size_t)kept].other);
        std::string err;
        if (cands[(size_t)kept].t) for (auto &c : cands[(size_t)kept].t->cond) attach(A, c, false, err);
    }
    // A_R = M_R * V_R: both conditions hold and both maps name the same unique index
    for (auto &a : mr)
        for (auto &b : vr) {
            if (!same_map(a, b, d)) continue;
            RedTerm t = a;
            for (auto &c : b.cond) t.cond.push_back(c);
            A.red.push_back(t);
        }
    return finish(A);
}

// ---- membership on the host (used by the inference of sums, which checks its candidates point by point) ----
static bool in_unique(const Desc &D, const i64 *x)
{
    if (D.empty) return false;
    for (int v = 0; v < D.d; ++v) {
        i64 l, h;
        range_of(D, v, x, l, h);
        if (x[v] < l || x[v] > h) return false;
    }
    return true;
}
// the unique index the redundancy map gives for x (x itself on the unique set); false where the tensor is zero
static bool unique_of(const Desc &D, const i64 *x, i64 *y)
{
    for (int v = 0; v < D.d; ++v) y[v] = x[v];
    if (in_unique(D, x)) return true;
    if (D.red_sort) {
        std::sort(y, y + D.d);
        if (in_unique(D, y)) return true;
    }
    for (auto &t : D.red) {
        bool ok = true;
        for (auto &c : t.cond) ok = ok && bound_eval(c, x, D.d) >= 0;
        if (!ok) continue;
        for (int v = 0; v < D.d; ++v) y[v] = bound_eval(t.map[v], x, D.d);
        if (in_unique(D, y)) return true;
    }
    return false;
}
template <typename F> static bool for_all_box(const Desc &D, F &&f)      // f(x) for every x of the box, until it returns false
{
    i64 x[MAXD] = {0, 0, 0, 0};
    i64 total = 1;
    for (int v = 0; v < D.d; ++v) total *= D.dims[v];
    for (i64 e = 0; e < total; ++e) {
        i64 r = e;
        for (int v = D.d - 1; v >= 0; --v) { x[v] = r % D.dims[v]; r /= D.dims[v]; }
        if (!f(x)) return false;
    }
    return true;
}

// A(x) := M(x) + V(x) ("Unique Set Inference": a sum is non-zero where either operand is, so the unique set of a
// sum is the union; "Redundancy Map Inference": operands of the SAME structure keep it, otherwise the
// redundancy maps are dropped first -- every non-zero element of an operand, unique or redundant, counts as
// stored -- and the result has none).  A descriptor holds one nest, so the union must be one: the candidates
// are the unique set of an operand without a redundancy map and the whole box, each checked point by point
// against the union of the two supports.
st_status infer_sum(const Desc &M, const Desc &V, Desc &A)
{
    if (M.d != V.d || !std::equal(M.dims, M.dims + MAXD, V.dims)) { A.error = "operands of different shape"; return ST_ERR_SHAPE; }
    const int d = M.d;
    i64 total = 1;
    for (int v = 0; v < d; ++v) total *= M.dims[v];
    if (total > ((i64)1 << 26)) { A.error = "the inference of a sum checks its result point by point: box above 2^26 elements"; return ST_ERR_UNSUPPORTED; }
    A.d = d; A.name = "A"; A.vars = M.vars;
    std::copy(M.dims, M.dims + MAXD, A.dims);
    // same structure: the same unique set and, off it, the same unique index
    const bool same = for_all_box(M, [&](const i64 *x) {
        i64 a[MAXD], b[MAXD];
        const bool ma = unique_of(M, x, a), vb = unique_of(V, x, b);
        return in_unique(M, x) == in_unique(V, x) && ma == vb && (!ma || std::equal(a, a + d, b));
    });
    if (same) {
        add_box(A, M);
        A.red = M.red;
        A.red_sort = M.red_sort;
        return finish(A);
    }
    auto support = [&](const i64 *x) { i64 y[MAXD]; return unique_of(M, x, y) || unique_of(V, x, y); };
    const Desc *cands[3] = {(M.red.empty() && !M.red_sort) ? &M : nullptr, (V.red.empty() && !V.red_sort) ? &V : nullptr, nullptr};
    for (int q = 0; q < 3; ++q) {
        if (q < 2 && !cands[q]) continue;
        const Desc *Cd = cands[q];
        const bool fits = for_all_box(M, [&](const i64 *x) { return (Cd ? in_unique(*Cd, x) : true) == support(x); });
        if (!fits) continue;
        if (Cd) add_box(A, *Cd);                 // (the whole box: no comparisons at all)
        return finish(A);
    }
    A.error = "the union of the two supports is neither an operand's unique set nor the whole box: a sum of nests";
    return ST_ERR_UNSUPPORTED;
}

// A(x_0..x_{d-2}) := sum over x_{d-1} of B(x): a rule head that leaves a variable of the body out sums over it
// ("marginalization"); "Unique Set Inference", projection: the output is non-zero where ANY value of the dropped
// variable is stored, i.e. where the run of that prefix is not empty.  With affine integer bounds and a unit
// coefficient on the dropped variable, "some x with every lower bound <= x <= every upper bound" is exactly
// "every lower bound <= every upper bound": one comparison among the earlier variables per pair of bounds.
// The packed order of the result is the run order of the operand.
st_status infer_project(const Desc &B, Desc &A)
{
    if (B.d < 2) { A.error = "nothing is left of an order-1 tensor"; return ST_ERR_SHAPE; }
    if (B.red_sort || !B.red.empty()) { A.error = "projection of an operand with a redundancy map is not supported"; return ST_ERR_UNSUPPORTED; }
    const int d = B.d - 1, last = B.d - 1;
    A.d = d;
    A.name = "A";
    for (int v = 0; v < d; ++v) { A.vars.push_back(B.vars[(size_t)v]); A.dims[v] = B.dims[v]; }
    Bound k;
    for (int u = 0; u < MAXD; ++u) k.coef[u] = 0;
    for (int v = 0; v < d; ++v) {
        k.c = B.first[v];
        A.lo[v].push_back(k);
        k.c = B.last[v];
        A.hi[v].push_back(k);
        for (auto &q : B.lo[v]) A.lo[v].push_back(q);
        for (auto &q : B.hi[v]) A.hi[v].push_back(q);
    }
    A.empty = B.empty;
    std::vector<Bound> los = B.lo[last], his = B.hi[last];
    k.c = B.first[last];
    los.push_back(k);
    k.c = B.last[last];
    his.push_back(k);
    for (auto &l : los)
        for (auto &h : his) {
            Bound c;                                       // h - l >= 0
            c.c = h.c - l.c;
            for (int u = 0; u < MAXD; ++u) c.coef[u] = h.coef[u] - l.coef[u];
            std::string err;
            if (!attach(A, c, false, err)) { A.error = "the comparison left by the dropped variable: " + err; return ST_ERR_UNSUPPORTED; }
        }
    return finish(A);
}

// Tensor outer product T(x, y) := M(x) * V(y) over disjoint index lists ("Redundancy Map Inference", outer
// product rule): T_U = M_U * V_U; T_R = M_U * V_R + M_R * V_U + M_R * V_R.  The variables of V follow those of M.
// A term of V alone maps the V part and keeps the M part (and the other way round); where both parts are
// redundant the first two lead outside the unique set and the combined term applies (the reconstruction tries
// the terms in order and takes the first whose target is stored).
static Bound shifted(const Bound &b, int by)
{
    Bound r;
    r.c = b.c;
    for (int u = 0; u < MAXD; ++u) r.coef[u] = 0;
    for (int u = 0; u + by < MAXD; ++u) r.coef[u + by] = b.coef[u];
    return r;
}
static Bound identity_map(int v)
{
    Bound r;
    r.c = 0;
    for (int u = 0; u < MAXD; ++u) r.coef[u] = u == v ? 1 : 0;
    return r;
}

st_status infer_outer(const Desc &M, const Desc &V, Desc &A)
{
    const int dm = M.d, dv = V.d, d = dm + dv;
    if (d > MAXD) { A.error = "the order of an outer product is limited to " + std::to_string(MAXD); return ST_ERR_UNSUPPORTED; }
    if ((M.red_sort && dm != 2) || (V.red_sort && dv != 2)) {
        A.error = "a 'sort' redundancy map of order above 2 is a sum of conditions: not supported in an outer product";
        return ST_ERR_UNSUPPORTED;
    }
    A.d = d;
    A.name = "T";
    for (int v = 0; v < dm; ++v) { A.vars.push_back(M.vars[(size_t)v]); A.dims[v] = M.dims[v]; }
    for (int v = 0; v < dv; ++v) {
        std::string name = V.vars[(size_t)v];
        while (std::find(A.vars.begin(), A.vars.end(), name) != A.vars.end()) name += "2";
        A.vars.push_back(name);
        A.dims[dm + v] = V.dims[v];
    }
    Desc Vs;                                              // V with its variables moved behind those of M
    Vs.d = d;
    for (int v = 0; v < dv; ++v) {
        Vs.first[dm + v] = V.first[v];
        Vs.last[dm + v] = V.last[v];
        for (auto &b : V.lo[v]) Vs.lo[dm + v].push_back(shifted(b, dm));
        for (auto &b : V.hi[v]) Vs.hi[dm + v].push_back(shifted(b, dm));
    }
    for (int v = 0; v < dm; ++v) { Vs.first[v] = 0; Vs.last[v] = M.dims[v] - 1; }
    Vs.empty = V.empty;
    add_box(A, M);                                        // (add_box walks S.d variables: the M part only)
    add_box(A, Vs);
    const std::vector<RedTerm> mr = terms_of(M), vr0 = terms_of(V);
    std::vector<RedTerm> vr;
    for (auto &t : vr0) {
        RedTerm q;
        for (int v = 0; v < MAXD; ++v) q.map[v] = identity_map(v);
        for (auto &c : t.cond) q.cond.push_back(shifted(c, dm));
        for (int v = 0; v < dv; ++v) q.map[dm + v] = shifted(t.map[v], dm);
        vr.push_back(q);
    }
    std::vector<RedTerm> mrx;
    for (auto &t : mr) {
        RedTerm q = t;
        for (int v = 0; v < dv; ++v) q.map[dm + v] = identity_map(dm + v);
        mrx.push_back(q);
    }
    for (auto &t : vr) A.red.push_back(t);                // M_U * V_R
    for (auto &t : mrx) A.red.push_back(t);               // M_R * V_U
    for (auto &a : mrx)                                   // M_R * V_R
        for (auto &b : vr) {
            RedTerm q;
            for (int v = 0; v < MAXD; ++v) q.map[v] = identity_map(v);
            q.cond = a.cond;
            for (auto &c : b.cond) q.cond.push_back(c);
            for (int v = 0; v < dm; ++v) q.map[v] = a.map[v];
            for (int v = 0; v < dv; ++v) q.map[dm + v] = b.map[dm + v];
            A.red.push_back(q);
        }
    return finish(A);
}

// k-fold outer product of a vector with itself, T(x_1..x_k) := v(x_1) * .. * v(x_k): the self-multiplication rule
// extended to higher degrees ("Extensions" of the inference rules; the vector self-outer-product example for
// k = 2): the unique set gains x_1 <= x_2 <= .. <= x_k on top of v's range on every index, every permutation of
// a stored tuple holds the same value (redundancy map: sort).  These are the structures of the covariance terms
// M1, M2, M3 of the overview.
st_status infer_power(const Desc &V, int k, Desc &A)
{
    if (V.d != 1) { A.error = "the self-product rule is implemented for vectors (order-1 descriptors)"; return ST_ERR_UNSUPPORTED; }
    if (k < 2 || k > MAXD) { A.error = "degree of the self product: 2.." + std::to_string(MAXD); return ST_ERR_SHAPE; }
    if (!V.red.empty() || V.red_sort) { A.error = "a vector with a redundancy map is not supported here"; return ST_ERR_UNSUPPORTED; }
    A.d = k;
    A.name = "T";
    const char *names[MAXD] = {"i", "j", "k", "l"};
    for (int v = 0; v < k; ++v) {
        A.vars.push_back(names[v]);
        A.dims[v] = V.dims[0];
        Bound b;
        for (int u = 0; u < MAXD; ++u) b.coef[u] = 0;
        b.c = V.first[0];
        A.lo[v].push_back(b);
        b.c = V.last[0];
        A.hi[v].push_back(b);
        if (v > 0) A.lo[v].push_back(identity_map(v - 1));         // x_v >= x_{v-1}
    }
    A.empty = V.empty;
    A.red_sort = true;
    return finish(A);
}

// Direct sum T := M (+) V ("Redundancy Map Inference", direct-sum rule; the top-right rule of "Representation of
// linear algebra operations"): with d = dims(M),
//     T_U(x)     := M_U(x) + V_U(y) * (y = x - d),
//     T_R(x, x') := M_R(x, x') + V_R(y, y') * (y = x - d) * (y' = x' - d).
// The two summands lie in disjoint boxes, so the unique set is a sum of two nests, and (as the paper's code
// generation gives every summand a nest of its own) each summand is returned as a descriptor of its own over the
// box of T: `place` writes the structure of S at offset `off` inside a box `dims` -- every bound, every condition
// and every map of S with x - off in the place of x.  The packed array of T is M_C followed by V_C; the shift
// keeps the nest order, so each part's packed order is the operand's.
st_status place(const Desc &S, const i64 *off, const i64 *dims, Desc &A)
{
    A.d = S.d;
    A.name = S.name;
    A.vars = S.vars;
    for (int v = 0; v < S.d; ++v) {
        if (off[v] < 0 || off[v] + S.dims[v] > dims[v]) { A.error = "the operand does not fit the box at this offset"; return ST_ERR_SHAPE; }
        if (S.red_sort && off[v] != off[0]) {
            A.error = "a 'sort' redundancy map needs the same offset on every index";
            return ST_ERR_UNSUPPORTED;
        }
        A.dims[v] = dims[v];
    }
    // value = c + sum coef[u] * x_u, read at x - off; `own` >= 0: the value is itself an index of variable `own`
    auto move = [&](const Bound &b, int own) {
        Bound r = b;
        for (int u = 0; u < S.d; ++u) r.c -= b.coef[u] * off[u];
        if (own >= 0) r.c += off[own];
        return r;
    };
    for (int v = 0; v < S.d; ++v) {
        Bound c;
        for (int u = 0; u < MAXD; ++u) c.coef[u] = 0;
        c.c = S.first[v] + off[v];
        A.lo[v].push_back(c);
        c.c = S.last[v] + off[v];
        A.hi[v].push_back(c);
        for (auto &b : S.lo[v]) A.lo[v].push_back(move(b, v));
        for (auto &b : S.hi[v]) A.hi[v].push_back(move(b, v));
    }
    A.empty = S.empty;
    A.red_sort = S.red_sort;
    for (auto &t : S.red) {
        RedTerm q;
        for (int v = 0; v < MAXD; ++v) q.map[v] = v < S.d ? move(t.map[v], v) : t.map[v];
        for (auto &c : t.cond) q.cond.push_back(move(c, -1));
        // the conditions of S were only ever read inside its own box
        for (int v = 0; v < S.d; ++v) {
            Bound in;
            for (int u = 0; u < MAXD; ++u) in.coef[u] = 0;
            in.coef[v] = 1;
            in.c = -off[v];
            q.cond.push_back(in);                                  // x_v - off_v >= 0
            in.coef[v] = -1;
            in.c = off[v] + S.dims[v] - 1;
            q.cond.push_back(in);                                  // off_v + dims_v - 1 - x_v >= 0
        }
        A.red.push_back(q);
    }
    return finish(A);
}

// the generated source compiled for gfx950 (no GPU needed); on failure D.error holds the compiler's log
st_status compile_source(Desc &D, std::vector<char> *code)
{
    hiprtcProgram prog;
    if (hiprtcCreateProgram(&prog, D.source.c_str(), "st_generated.hip", 0, nullptr, nullptr) != HIPRTC_SUCCESS)
        return ST_ERR_LAUNCH;
    const char *opts[] = {"--offload-arch=gfx950", "-O3", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"};
    const hiprtcResult rc = hiprtcCompileProgram(prog, 6, opts);
    if (rc != HIPRTC_SUCCESS) {
        size_t n = 0;
        hiprtcGetProgramLogSize(prog, &n);
        std::string log(n, '\0');
        if (n) hiprtcGetProgramLog(prog, &log[0]);
        D.error = "hiprtc: " + log;
    } else if (code) {
        size_t n = 0;
        hiprtcGetCodeSize(prog, &n);
        code->resize(n);
        hiprtcGetCode(prog, code->data());
    }
    hiprtcDestroyProgram(&prog);
    return rc == HIPRTC_SUCCESS ? ST_OK : ST_ERR_LAUNCH;
}

// compile the generated source for the current device and load it (once per device)
st_status module_for(Desc &D, Desc::Loaded &out)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return ST_ERR_LAUNCH;
    std::lock_guard<std::mutex> lock(D.mu);
    auto it = D.modules.find(dev);
    if (it != D.modules.end()) { out = it->second; return ST_OK; }
    std::vector<char> code;
    if (compile_source(D, &code) != ST_OK) return ST_ERR_LAUNCH;
    Desc::Loaded L;
    if (hipModuleLoadData(&L.mod, code.data()) != hipSuccess) { D.error = "hipModuleLoadData failed"; return ST_ERR_LAUNCH; }
    const char *names[6] = {"st_gen_list", "st_gen_thp", "st_gen_expand", "st_gen_gather", "st_gen_moment",
                            "st_gen_moment_reduce"};
    L.fn[4] = L.fn[5] = L.fn[6] = L.fn[7] = L.fn[8] = nullptr;
    for (int q = 0; q < 10; ++q) {
        if ((q == 4 || q == 5) && D.ntiles == 0) continue;      // moment kernels: equal extents only
        if ((q == 6 || q == 7) && D.d != 3) continue;           // MTTKRP: order 3 only
        const char *name = q == 6 ? "st_gen_mttkrp" : q == 7 ? "st_gen_mttkrp_combine" : q == 8 ? "st_gen_sum_last"
                         : q == 9 ? "st_gen_expand_onto" : names[q];
        if (hipModuleGetFunction(&L.fn[q], L.mod, name) != hipSuccess) {
            (void)hipModuleUnload(L.mod);
            D.error = std::string("generated kernel missing: ") + name;
            return ST_ERR_LAUNCH;
        }
    }
    D.modules[dev] = L;
    out = L;
    return ST_OK;
}

st_status launch_generated(Desc &D, int which, unsigned blocks, void **args, hipStream_t s, unsigned gy = 1,
                           unsigned threads = 256, unsigned lds_bytes = 0)
{
    if (blocks == 0 || gy == 0) return ST_OK;
    Desc::Loaded L;
    st_status rc = module_for(D, L);
    if (rc != ST_OK) return rc;
    if (hipModuleLaunchKernel(L.fn[which], blocks, gy, 1, threads, 1, 1, lds_bytes, s, args, nullptr) != hipSuccess)
        return ST_ERR_LAUNCH;
    return ST_OK;
}

// sample slices and chunk size of the generated moment kernels
struct MomentPlan { unsigned threads, gx, ch, S; i64 slice; };
MomentPlan moment_plan(const Desc &D, i64 N)
{
    MomentPlan p;
    p.threads = D.ntiles >= 256 ? 256u : (unsigned)((D.ntiles + 63) / 64) * 64u;
    p.gx = (unsigned)((D.ntiles + p.threads - 1) / p.threads);
    unsigned ch = (unsigned)(8192 / D.mnp);                  // two chunks of at most 8192 floats: 64 KB of LDS
    p.ch = ch > 64u ? 64u : ch & ~3u;
    i64 S = (1024 + p.gx - 1) / p.gx;
    const i64 smax = (N + p.ch - 1) / p.ch;
    if (S > smax) S = smax;
    if (S > 1024) S = 1024;
    if (S < 1) S = 1;
    p.slice = ((N + S - 1) / S + p.ch - 1) / p.ch * p.ch;
    p.S = (unsigned)((N + p.slice - 1) / p.slice);
    return p;
}

}  // namespace
}  // namespace st

using namespace st;

extern "C" {

st_status st_desc_create(const char *unique_set, const char *redundancy, const int64_t *dims, int ndims,
                         const char *const *param_names, const int64_t *param_values, int nparams, st_desc **out)
{
    if (!unique_set || !dims || !out || (nparams > 0 && (!param_names || !param_values))) return ST_ERR_NULL;
    if (ndims < 1 || ndims > MAXD || nparams < 0) return ST_ERR_SHAPE;
    Desc *D = new Desc();
    st_status rc = parse_all(*D, unique_set, redundancy, dims, ndims, param_names, param_values, nparams);
    *out = reinterpret_cast<st_desc *>(D);     // kept on failure too: st_desc_error tells why
    return rc;
}

void st_desc_destroy(st_desc *desc)
{
    Desc *D = reinterpret_cast<Desc *>(desc);
    if (!D) return;
    for (auto &kv : D->modules) (void)hipModuleUnload(kv.second.mod);
    delete D;
}

const char *st_desc_error(const st_desc *desc) { return desc ? reinterpret_cast<const Desc *>(desc)->error.c_str() : ""; }
int64_t st_desc_count(const st_desc *desc) { return desc ? reinterpret_cast<const Desc *>(desc)->count : -1; }
int64_t st_desc_runs(const st_desc *desc) { return desc ? reinterpret_cast<const Desc *>(desc)->nruns : -1; }
const char *st_desc_nest(const st_desc *desc) { return desc ? reinterpret_cast<const Desc *>(desc)->nest.c_str() : ""; }
const char *st_desc_source(const st_desc *desc) { return desc ? reinterpret_cast<const Desc *>(desc)->source.c_str() : ""; }
size_t st_desc_table_bytes(const st_desc *desc)
{
    return desc ? reinterpret_cast<const Desc *>(desc)->table.size() * sizeof(int32_t) : 0;
}

st_status st_desc_table(const st_desc *desc, void *host_out)
{
    if (!desc || !host_out) return ST_ERR_NULL;
    const Desc *D = reinterpret_cast<const Desc *>(desc);
    memcpy(host_out, D->table.data(), D->table.size() * sizeof(int32_t));
    return ST_OK;
}

st_status st_desc_compile(st_desc *desc)
{
    if (!desc) return ST_ERR_NULL;
    Desc *D = reinterpret_cast<Desc *>(desc);
    if (D->source.empty()) return ST_ERR_SHAPE;
    return compile_source(*D, nullptr);
}

st_status st_desc_list(st_desc *desc, const void *table, int32_t *out, void *stream)
{
    if (!desc || !table || !out) return ST_ERR_NULL;
    Desc *D = reinterpret_cast<Desc *>(desc);
    if (D->source.empty()) return ST_ERR_SHAPE;
    if (!aligned16(table) || !aligned16(out)) return ST_ERR_ALIGN;
    void *args[] = {&table, &out};
    return launch_generated(*D, 0, (unsigned)((D->nruns + 3) / 4), args, (hipStream_t)stream);
}

st_status st_desc_thp(st_desc *desc, const void *table, const float *Bc, const float *C, float *Ac, void *stream)
{
    if (!desc || !table || !Bc || !C || !Ac) return ST_ERR_NULL;
    Desc *D = reinterpret_cast<Desc *>(desc);
    if (D->source.empty()) return ST_ERR_SHAPE;
    if (!aligned16(table) || !aligned16(Bc) || !aligned16(C) || !aligned16(Ac)) return ST_ERR_ALIGN;
    size_t pb = (size_t)D->count * 4, cb = (size_t)D->prefixes * D->dims[D->d - 1] * 4;
    if (overlap(Ac, pb, Bc, pb) || overlap(Ac, pb, C, cb)) return ST_ERR_SHAPE;
    void *args[] = {&table, &Bc, &C, &Ac};
    return launch_generated(*D, 1, (unsigned)((D->nruns + 3) / 4), args, (hipStream_t)stream);
}

// every run of the unique set is a whole fibre of the last variable
static bool last_variable_free(const Desc &D)
{
    const int last = D.d - 1;
    return D.d >= 2 && D.lo[last].empty() && D.hi[last].empty() && D.first[last] == 0 && D.last[last] == D.dims[last] - 1;
}

size_t st_desc_mttkrp_workspace(const st_desc *desc, int R)
{
    if (!desc || R < 1) return 0;
    const Desc *D = reinterpret_cast<const Desc *>(desc);
    if (D->d != 3 || D->source.empty() || !last_variable_free(*D) || D->nruns == 0) return 0;
    return ((size_t)D->nruns * (size_t)R * sizeof(float) + 255u) & ~(size_t)255u;          // Y(run, r)
}

st_status st_desc_mttkrp(st_desc *desc, const void *table, const float *Bc, const float *C, const float *Dm, float *A,
                         int R, void *ws, size_t ws_bytes, void *stream)
{
    if (!desc || !table || !Bc || !C || !Dm || !A) return ST_ERR_NULL;
    Desc *D = reinterpret_cast<Desc *>(desc);
    if (D->source.empty() || R < 1) return ST_ERR_SHAPE;
    // order 3, sparsity structures only: with a redundancy map the operand has entries outside its unique set
    if (D->d != 3 || D->red_sort || !D->red.empty()) return ST_ERR_UNSUPPORTED;
    if ((int64_t)R * std::max(D->dims[1], D->dims[2]) > ((int64_t)1 << 31) || D->dims[0] > 0x7fffffff) return ST_ERR_UNSUPPORTED;
    if (!aligned16(table) || !aligned16(Bc) || !aligned16(C) || !aligned16(Dm) || !aligned16(A)) return ST_ERR_ALIGN;
    const size_t bb = (size_t)D->count * 4, cb = (size_t)D->dims[1] * R * 4, db = (size_t)D->dims[2] * R * 4,
                 ab = (size_t)D->dims[0] * R * 4;
    if (overlap(A, ab, Bc, bb) || overlap(A, ab, C, cb) || overlap(A, ab, Dm, db)) return ST_ERR_SHAPE;
    const size_t need = st_desc_mttkrp_workspace(desc, R);
    if (need > 0) {
        // last variable free: the contraction over it runs on the matrix cores (the fibres of the unique set are the
        // rows of a plain matrix), then the runs of every output row are combined with the rows of C
        if (!ws || ws_bytes < need) return ST_ERR_WORKSPACE;
        if (!aligned16(ws)) return ST_ERR_ALIGN;
        if (overlap(ws, need, Bc, bb) || overlap(ws, need, C, cb) || overlap(ws, need, Dm, db) || overlap(ws, need, A, ab))
            return ST_ERR_SHAPE;
        if ((int64_t)D->nruns * R > ((int64_t)1 << 40)) return ST_ERR_UNSUPPORTED;
        float *Y = static_cast<float *>(ws);
        const st_status rc = launch_ttm(Bc, Dm, Y, D->nruns, (int)D->dims[2], R, nullptr, (hipStream_t)stream);
        if (rc != ST_OK) return rc;
        const float *Yc = Y;
        void *args[] = {&table, &Yc, &C, &A, &R};
        const unsigned threads = D->dims[1] >= 16 ? 1024u : 256u;             // 16 or 4 run slots of 64 columns
        return launch_generated(*D, 7, (unsigned)D->dims[0], args, (hipStream_t)stream, (unsigned)((R + 63) / 64), threads);
    }
    void *args[] = {&table, &Bc, &C, &Dm, &A, &R};
    // the runs of a row are a serial chain of dependent loads per wave: long rows get sixteen waves
    const unsigned threads = D->dims[1] >= 64 ? 1024u : 256u;
    return launch_generated(*D, 6, (unsigned)D->dims[0], args, (hipStream_t)stream, (unsigned)((R + 15) / 16), threads);
}

st_status st_desc_ttm(st_desc *desc, const float *Bc, const float *U, float *Ac, int R, void *stream)
{
    if (!desc || !Bc || !U || !Ac) return ST_ERR_NULL;
    Desc *D = reinterpret_cast<Desc *>(desc);
    if (D->source.empty() || R < 1) return ST_ERR_SHAPE;
    const int last = D->d - 1;
    // the contracted (last) variable must be free: every run is a whole fibre
    if (!last_variable_free(*D)) return ST_ERR_UNSUPPORTED;
    if (!aligned16(Bc) || !aligned16(U) || !aligned16(Ac)) return ST_ERR_ALIGN;
    const int64_t rows = D->nruns, nl = D->dims[last];
    if (nl * (int64_t)R > ((int64_t)1 << 31)) return ST_ERR_UNSUPPORTED;
    size_t tb = (size_t)rows * nl * 4, ub = (size_t)nl * R * 4, yb = (size_t)rows * R * 4;
    if (overlap(Ac, yb, Bc, tb) || overlap(Ac, yb, U, ub)) return ST_ERR_SHAPE;
    return launch_ttm(Bc, U, Ac, rows, (int)nl, R, nullptr, (hipStream_t)stream);
}

size_t st_desc_moment_workspace(const st_desc *desc, int64_t N)
{
    if (!desc || N <= 0) return 0;
    const Desc *D = reinterpret_cast<const Desc *>(desc);
    if (D->ntiles == 0) return 0;
    const MomentPlan p = moment_plan(*D, N);
    return (size_t)p.S * (size_t)D->ntiles * 64u * sizeof(float);
}

st_status st_desc_moment(st_desc *desc, const void *table, const float *X, int64_t N, float *Sc, int accumulate,
                         void *ws, size_t ws_bytes, void *stream)
{
    if (!desc || !table || !Sc || (N > 0 && !X)) return ST_ERR_NULL;
    Desc *D = reinterpret_cast<Desc *>(desc);
    if (D->source.empty() || N < 0 || (accumulate != 0 && accumulate != 1)) return ST_ERR_SHAPE;
    if (D->mbs == 0) return ST_ERR_UNSUPPORTED;      /* order 2 or 3 with equal extents <= 256 only */
    if (!aligned16(table) || !aligned16(Sc) || (X && !aligned16(X))) return ST_ERR_ALIGN;
    const size_t sb = (size_t)D->count * 4, xb = (size_t)N * D->dims[0] * 4;
    if (N > 0 && overlap(Sc, sb, X, xb)) return ST_ERR_SHAPE;
    if (D->ntiles == 0) return ST_OK;                /* empty unique set */
    if (N == 0) {           /* overwrite: the reduce kernel over zero slices writes the zeros */
        if (accumulate) return ST_OK;
        int S0 = 0;
        const void *none = table;
        void *a0[] = {&table, &none, &S0, &Sc, &accumulate};
        return launch_generated(*D, 5, (unsigned)((D->ntiles * 64 + 15) / 16), a0, (hipStream_t)stream);
    }
    const size_t need = st_desc_moment_workspace(desc, N);
    if (!ws || ws_bytes < need) return ST_ERR_WORKSPACE;
    if (!aligned16(ws)) return ST_ERR_ALIGN;
    if (overlap(ws, need, Sc, sb) || overlap(ws, need, X, xb)) return ST_ERR_SHAPE;
    const MomentPlan p = moment_plan(*D, N);
    long long Nll = N, slice = p.slice;
    int ch = (int)p.ch, S = (int)p.S;
    void *a1[] = {&table, &X, &Nll, &ch, &slice, &ws};
    st_status rc = launch_generated(*D, 4, p.gx, a1, (hipStream_t)stream, p.S, p.threads,
                                    (unsigned)(2u * p.ch * D->mnp * sizeof(float)));
    if (rc != ST_OK) return rc;
    void *a2[] = {&table, &ws, &S, &Sc, &accumulate};
    return launch_generated(*D, 5, (unsigned)((D->ntiles * 64 + 15) / 16), a2, (hipStream_t)stream);
}

st_status st_desc_product(const st_desc *m, const st_desc *v, st_desc **out)
{
    if (!m || !v || !out) return ST_ERR_NULL;
    const Desc *M = reinterpret_cast<const Desc *>(m), *V = reinterpret_cast<const Desc *>(v);
    if (M->source.empty() || V->source.empty()) return ST_ERR_SHAPE;
    Desc *A = new Desc();
    const st_status rc = infer_product(*M, *V, *A);
    *out = reinterpret_cast<st_desc *>(A);      // kept on failure too: st_desc_error tells why
    return rc;
}

st_status st_desc_outer(const st_desc *m, const st_desc *v, st_desc **out)
{
    if (!m || !v || !out) return ST_ERR_NULL;
    const Desc *M = reinterpret_cast<const Desc *>(m), *V = reinterpret_cast<const Desc *>(v);
    if (M->source.empty() || V->source.empty()) return ST_ERR_SHAPE;
    Desc *A = new Desc();
    const st_status rc = infer_outer(*M, *V, *A);
    *out = reinterpret_cast<st_desc *>(A);      // kept on failure too: st_desc_error tells why
    return rc;
}

st_status st_desc_sum(const st_desc *m, const st_desc *v, st_desc **out)
{
    if (!m || !v || !out) return ST_ERR_NULL;
    const Desc *M = reinterpret_cast<const Desc *>(m), *V = reinterpret_cast<const Desc *>(v);
    if (M->source.empty() || V->source.empty()) return ST_ERR_SHAPE;
    Desc *A = new Desc();
    const st_status rc = infer_sum(*M, *V, *A);
    *out = reinterpret_cast<st_desc *>(A);
    return rc;
}

st_status st_desc_project(const st_desc *b, st_desc **out)
{
    if (!b || !out) return ST_ERR_NULL;
    const Desc *B = reinterpret_cast<const Desc *>(b);
    if (B->source.empty()) return ST_ERR_SHAPE;
    Desc *A = new Desc();
    const st_status rc = infer_project(*B, *A);
    *out = reinterpret_cast<st_desc *>(A);
    return rc;
}

st_status st_desc_sum_last(st_desc *desc, const void *table, const float *Bc, float *out, void *stream)
{
    if (!desc || !table || !Bc || !out) return ST_ERR_NULL;
    Desc *D = reinterpret_cast<Desc *>(desc);
    if (D->source.empty()) return ST_ERR_SHAPE;
    if (D->red_sort || !D->red.empty()) return ST_ERR_UNSUPPORTED;
    if (!aligned16(table) || !aligned16(Bc) || !aligned16(out)) return ST_ERR_ALIGN;
    if (overlap(out, (size_t)D->nruns * 4, Bc, (size_t)D->count * 4)) return ST_ERR_SHAPE;
    void *args[] = {&table, &Bc, &out};
    return launch_generated(*D, 8, (unsigned)((D->nruns + 3) / 4), args, (hipStream_t)stream);
}

st_status st_desc_power(const st_desc *v, int k, st_desc **out)
{
    if (!v || !out) return ST_ERR_NULL;
    const Desc *V = reinterpret_cast<const Desc *>(v);
    if (V->source.empty()) return ST_ERR_SHAPE;
    Desc *A = new Desc();
    const st_status rc = infer_power(*V, k, *A);
    *out = reinterpret_cast<st_desc *>(A);
    return rc;
}

st_status st_desc_direct_sum(const st_desc *m, const st_desc *v, st_desc **out_m, st_desc **out_v)
{
    if (!m || !v || !out_m || !out_v) return ST_ERR_NULL;
    *out_m = *out_v = nullptr;
    const Desc *M = reinterpret_cast<const Desc *>(m), *V = reinterpret_cast<const Desc *>(v);
    if (M->source.empty() || V->source.empty() || M->d != V->d) return ST_ERR_SHAPE;
    i64 dims[MAXD] = {0, 0, 0, 0}, zero[MAXD] = {0, 0, 0, 0};
    for (int q = 0; q < M->d; ++q) dims[q] = M->dims[q] + V->dims[q];
    Desc *A = new Desc();
    st_status rc = place(*M, zero, dims, *A);
    *out_m = reinterpret_cast<st_desc *>(A);      // kept on failure too: st_desc_error tells why
    if (rc != ST_OK) return rc;
    Desc *B = new Desc();
    rc = place(*V, M->dims, dims, *B);
    *out_v = reinterpret_cast<st_desc *>(B);
    return rc;
}

st_status st_desc_expand_onto(st_desc *desc, const void *table, const float *Tc, float *T, void *stream)
{
    if (!desc || !table || !Tc || !T) return ST_ERR_NULL;
    Desc *D = reinterpret_cast<Desc *>(desc);
    if (D->source.empty()) return ST_ERR_SHAPE;
    if (!aligned16(table) || !aligned16(Tc) || !aligned16(T)) return ST_ERR_ALIGN;
    const int64_t total = D->prefixes * D->dims[D->d - 1];
    if (overlap(T, (size_t)total * 4, Tc, (size_t)D->count * 4)) return ST_ERR_SHAPE;
    void *args[] = {&table, &Tc, &T};
    return launch_generated(*D, 9, (unsigned)((total + 255) / 256), args, (hipStream_t)stream);
}

st_status st_desc_gather(st_desc *desc, const void *table, const float *Tc, const int32_t *idx, int64_t count,
                         int idx_stride, int idx_offset, const float *scale, const float *addend, float *out,
                         void *stream)
{
    if (!desc || !table || !Tc || (count > 0 && (!idx || !out))) return ST_ERR_NULL;
    Desc *D = reinterpret_cast<Desc *>(desc);
    if (D->source.empty() || count < 0) return ST_ERR_SHAPE;
    if (idx_offset < 0 || idx_stride < idx_offset + D->d || idx_stride > 64) return ST_ERR_SHAPE;
    if (count > ((int64_t)1 << 31) * 200) return ST_ERR_UNSUPPORTED;
    if (!aligned16(table) || !aligned16(Tc) || !aligned16(idx) || !aligned16(out) || (scale && !aligned16(scale)) ||
        (addend && !aligned16(addend)))
        return ST_ERR_ALIGN;
    if (count == 0) return ST_OK;
    if (overlap(out, (size_t)count * 4, Tc, (size_t)D->count * 4) ||
        overlap(out, (size_t)count * 4, idx, (size_t)count * 4 * (size_t)idx_stride))
        return ST_ERR_SHAPE;
    long long cnt = count;
    void *args[] = {&table, &Tc, &idx, &cnt, &idx_stride, &idx_offset, &scale, &addend, &out};
    return launch_generated(*D, 3, (unsigned)((count + 255) / 256), args, (hipStream_t)stream);
}

st_status st_desc_expand(st_desc *desc, const void *table, const float *Tc, float *T, void *stream)
{
    if (!desc || !table || !Tc || !T) return ST_ERR_NULL;
    Desc *D = reinterpret_cast<Desc *>(desc);
    if (D->source.empty()) return ST_ERR_SHAPE;
    if (!aligned16(table) || !aligned16(Tc) || !aligned16(T)) return ST_ERR_ALIGN;
    const int64_t total = D->prefixes * D->dims[D->d - 1];
    if (overlap(T, (size_t)total * 4, Tc, (size_t)D->count * 4)) return ST_ERR_SHAPE;
    void *args[] = {&table, &Tc, &T};
    const int64_t threads = D->dims[D->d - 1] % 4 == 0 ? total / 4 : total;     // as in the generated kernel
    return launch_generated(*D, 2, (unsigned)((threads + 255) / 256), args, (hipStream_t)stream);
}

}  // extern "C"
