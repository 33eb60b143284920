// Terms, the two term languages, their rewrite rules, the strategy-expression compiler and the
// lowering of a scheduled loop nest to a kernel configuration.  See elevate.hpp.  Host code only.
#include "elevate.hpp"

#include <cctype>
#include <cstdlib>
#include <set>

namespace elevate {

// ---- terms: equality, printing, parsing ------------------------------------------------------------
bool equal(const TermP &a, const TermP &b)
{
    if (a.get() == b.get()) return true;
    if (a->compound != b->compound || a->head != b->head || a->args.size() != b->args.size()) return false;
    for (size_t i = 0; i < a->args.size(); ++i)
        if (!equal(a->args[i], b->args[i])) return false;
    return true;
}

std::string print(const TermP &t)
{
    if (!t->compound) return t->head;
    std::string s = "(" + t->head;
    for (const auto &a : t->args) s += " " + print(a);
    return s + ")";
}

namespace {

struct Parser {
    const std::string &text;
    size_t pos;
    std::string err;
    void skip()
    {
        while (pos < text.size()) {
            if (std::isspace((unsigned char)text[pos])) {
                ++pos;
            } else if (text[pos] == ';') {                 // comment to the end of the line
                while (pos < text.size() && text[pos] != '\n') ++pos;
            } else {
                break;
            }
        }
    }
    std::string token()
    {
        size_t start = pos;
        while (pos < text.size() && !std::isspace((unsigned char)text[pos]) && text[pos] != '(' && text[pos] != ')' &&
               text[pos] != ';')
            ++pos;
        return text.substr(start, pos - start);
    }
    TermP term(int depth)
    {
        if (depth > 2000) { err = "nesting too deep"; return nullptr; }
        skip();
        if (pos >= text.size()) { err = "unexpected end of input"; return nullptr; }
        if (text[pos] == ')') { err = "unexpected ')'"; return nullptr; }
        if (text[pos] != '(') {
            std::string tok = token();
            if (tok.empty()) { err = "empty token"; return nullptr; }
            return atom(tok);
        }
        ++pos;
        skip();
        if (pos >= text.size() || text[pos] == '(' || text[pos] == ')') { err = "a list starts with a head symbol"; return nullptr; }
        std::string head = token();
        std::vector<TermP> args;
        for (;;) {
            skip();
            if (pos >= text.size()) { err = "missing ')'"; return nullptr; }
            if (text[pos] == ')') { ++pos; break; }
            TermP a = term(depth + 1);
            if (!a) return nullptr;
            args.push_back(a);
        }
        return node(head, std::move(args));
    }
};

bool parse_int(const TermP &t, long long &v)
{
    if (!is_atom(t) || t->head.empty()) return false;
    char *end = nullptr;
    v = std::strtoll(t->head.c_str(), &end, 10);
    return *end == '\0';
}

TermP int_atom(long long v) { return atom(std::to_string(v)); }

}  // namespace

TermP parse(const std::string &text, std::string &err)
{
    Parser p{text, 0, std::string()};
    TermP t = p.term(0);
    if (t) {
        p.skip();
        if (p.pos != text.size()) { err = "trailing input after the term"; return nullptr; }
    } else {
        err = p.err;
    }
    return t;
}

// ---- trace and rules ---------------------------------------------------------------------------------
Trace *&current_trace()
{
    static thread_local Trace *t = nullptr;
    return t;
}

Strategy<TermP> rule(const std::string &name, std::function<TermP(const TermP &)> fn)
{
    return Strategy<TermP>(name, [name, fn](const TermP &p) {
        Trace *tr = current_trace();
        if (tr && tr->steps.size() >= tr->limit) {
            tr->exhausted = true;                       // every rule now fails, so every repeat ends
            return RewriteResult<TermP>::failure(name);
        }
        TermP q = fn(p);
        if (!q) return RewriteResult<TermP>::failure(name);
        if (tr) tr->steps.push_back(Trace::Step{name, print(p), print(q)});
        return RewriteResult<TermP>::success(q);
    });
}

// ---- the functional array language of Section 4 -------------------------------------------------------
// (let x e0 e1)  (fun x e)  (app f a)  (build n f)  (get a i)  (length a); atoms are variables and
// integer literals.
namespace {

void free_vars(const TermP &e, std::set<std::string> &bound, std::set<std::string> &out)
{
    if (is_atom(e)) {
        if (!bound.count(e->head)) out.insert(e->head);
        return;
    }
    if (is_node(e, "fun", 2) && is_atom(e->args[0])) {
        const std::string &x = e->args[0]->head;
        const bool was = bound.count(x) > 0;
        bound.insert(x);
        free_vars(e->args[1], bound, out);
        if (!was) bound.erase(x);
        return;
    }
    if (is_node(e, "let", 3) && is_atom(e->args[0])) {
        free_vars(e->args[1], bound, out);
        const std::string &x = e->args[0]->head;
        const bool was = bound.count(x) > 0;
        bound.insert(x);
        free_vars(e->args[2], bound, out);
        if (!was) bound.erase(x);
        return;
    }
    for (const auto &a : e->args) free_vars(a, bound, out);
}

std::set<std::string> free_vars(const TermP &e)
{
    std::set<std::string> bound, out;
    free_vars(e, bound, out);
    return out;
}

// a name based on y that is in none of the given sets
std::string fresh_name(const std::string &y, const std::set<std::string> &avoid)
{
    std::string z = y;
    do { z += "'"; } while (avoid.count(z));
    return z;
}

}  // namespace

TermP substitute(const TermP &e, const std::string &x, const TermP &v)
{
    if (is_atom(e)) return e->head == x ? v : e;
    const bool is_fun = is_node(e, "fun", 2) && is_atom(e->args[0]);
    const bool is_let = is_node(e, "let", 3) && is_atom(e->args[0]);
    if (is_fun || is_let) {
        std::string y = e->args[0]->head;
        TermP scope = e->args[is_fun ? 1 : 2];            // where y is bound
        TermP bound_to = is_let ? substitute(e->args[1], x, v) : nullptr;
        if (y != x) {
            const std::set<std::string> fv = free_vars(v);
            if (fv.count(y) && free_vars(scope).count(x)) {
                // y would capture a free variable of v: rename the binder first
                std::set<std::string> avoid = fv;
                const std::set<std::string> fs = free_vars(scope);
                avoid.insert(fs.begin(), fs.end());
                avoid.insert(x);
                const std::string y2 = fresh_name(y, avoid);
                scope = substitute(scope, y, atom(y2));
                y = y2;
            }
            scope = substitute(scope, x, v);
        }
        if (is_fun) return node("fun", {atom(y), scope});
        return node("let", {atom(y), bound_to, scope});
    }
    std::vector<TermP> args;
    args.reserve(e->args.size());
    for (const auto &a : e->args) args.push_back(substitute(a, x, v));
    return node(e->head, std::move(args));
}

namespace {

bool alpha_eq(const TermP &a, const TermP &b, std::vector<std::pair<std::string, std::string>> &env)
{
    if (is_atom(a) || is_atom(b)) {
        if (!is_atom(a) || !is_atom(b)) return false;
        for (size_t i = env.size(); i-- > 0;) {
            const bool la = env[i].first == a->head, lb = env[i].second == b->head;
            if (la || lb) return la && lb;                // innermost binder of either name decides
        }
        return a->head == b->head;                        // both free
    }
    if (a->head != b->head || a->args.size() != b->args.size()) return false;
    const bool is_fun = is_node(a, "fun", 2) && is_atom(a->args[0]) && is_atom(b->args[0]);
    const bool is_let = is_node(a, "let", 3) && is_atom(a->args[0]) && is_atom(b->args[0]);
    if (is_fun || is_let) {
        if (is_let && !alpha_eq(a->args[1], b->args[1], env)) return false;
        env.emplace_back(a->args[0]->head, b->args[0]->head);
        const bool r = alpha_eq(a->args[is_fun ? 1 : 2], b->args[is_fun ? 1 : 2], env);
        env.pop_back();
        return r;
    }
    for (size_t i = 0; i < a->args.size(); ++i)
        if (!alpha_eq(a->args[i], b->args[i], env)) return false;
    return true;
}

}  // namespace

bool alpha_equal(const TermP &a, const TermP &b)
{
    std::vector<std::pair<std::string, std::string>> env;
    return alpha_eq(a, b, env);
}

namespace {

// Section 4, fusion rules:  (build e0 e1)[e2] ~> e1 e2      length (build e0 e1) ~> e0
Strategy<TermP> buildGet()
{
    return rule("buildGet", [](const TermP &p) -> TermP {
        if (is_node(p, "get", 2) && is_node(p->args[0], "build", 2)) return node("app", {p->args[0]->args[1], p->args[1]});
        return nullptr;
    });
}
Strategy<TermP> lenBuild()
{
    return rule("lenBuild", [](const TermP &p) -> TermP {
        if (is_node(p, "length", 1) && is_node(p->args[0], "build", 2)) return p->args[0]->args[0];
        return nullptr;
    });
}
// partial evaluation of a binding: let x = e0 in e1 ~> e1[x := e0]
Strategy<TermP> letPartialEval()
{
    return rule("letPartialEval", [](const TermP &p) -> TermP {
        if (is_node(p, "let", 3) && is_atom(p->args[0])) return substitute(p->args[2], p->args[0]->head, p->args[1]);
        return nullptr;
    });
}
// a binding in function position moves outwards: (let x = e0 in e1) e2 ~> let x = e0 in (e1 e2)
Strategy<TermP> letApp()
{
    return rule("letApp", [](const TermP &p) -> TermP {
        if (!(is_node(p, "app", 2) && is_node(p->args[0], "let", 3) && is_atom(p->args[0]->args[0]))) return nullptr;
        const TermP &let = p->args[0];
        std::string x = let->args[0]->head;
        TermP e1 = let->args[2];
        const std::set<std::string> fv2 = free_vars(p->args[1]);
        if (fv2.count(x)) {                                // keep e2's x out of the binding's scope
            std::set<std::string> avoid = fv2;
            const std::set<std::string> f1 = free_vars(e1);
            avoid.insert(f1.begin(), f1.end());
            const std::string x2 = fresh_name(x, avoid);
            e1 = substitute(e1, x, atom(x2));
            x = x2;
        }
        return node("let", {atom(x), let->args[1], node("app", {e1, p->args[1]})});
    });
}
// application of a function literal becomes a binding: (fun x -> e) v ~> let x = v in e
Strategy<TermP> funToLet()
{
    return rule("funToLet", [](const TermP &p) -> TermP {
        if (is_node(p, "app", 2) && is_node(p->args[0], "fun", 2) && is_atom(p->args[0]->args[0]))
            return node("let", {p->args[0]->args[0], p->args[1], p->args[0]->args[1]});
        return nullptr;
    });
}

// ---- the loop-nest language: (loop AXIS EXTENT KIND BODY), leaves mac and mfma32x32x2 ------------------
// AXIS is M, N or K of the product; KIND is seq, grid (one workgroup per iteration), wave (one wave
// per iteration), unroll (register-blocked, fully unrolled) or slab (a K loop whose every iteration
// stages one slab of both operands through LDS).
struct Loop { std::string axis; long long extent; std::string kind; TermP body; };

bool as_loop(const TermP &t, Loop &l)
{
    if (!is_node(t, "loop", 4) || !is_atom(t->args[0]) || !is_atom(t->args[2])) return false;
    if (!parse_int(t->args[1], l.extent) || l.extent < 1) return false;
    l.axis = t->args[0]->head;
    l.kind = t->args[2]->head;
    l.body = t->args[3];
    return l.axis == "M" || l.axis == "N" || l.axis == "K";
}
TermP make_loop(const std::string &axis, long long extent, const std::string &kind, const TermP &body)
{
    return node("loop", {atom(axis), int_atom(extent), atom(kind), body});
}

// Loop blocking (strip-mining), the split of Section 6.2 for a loop instead of a map: a sequential
// loop of extent E over `axis` becomes ceil(E/n) iterations of a loop of extent n.
Strategy<TermP> split(const std::string &axis, long long n)
{
    return rule("split(" + axis + "," + std::to_string(n) + ")", [axis, n](const TermP &p) -> TermP {
        Loop l;
        if (!as_loop(p, l) || l.axis != axis || l.kind != "seq" || l.extent <= n) return nullptr;
        return make_loop(axis, (l.extent + n - 1) / n, "seq", make_loop(axis, n, "seq", l.body));
    });
}
// Rounds the extent of a sequential loop up to a multiple of n: the iterations added compute on
// zero-filled operands and their results are masked (how the kernels treat ragged edges).
Strategy<TermP> cover(const std::string &axis, long long n)
{
    return rule("cover(" + axis + "," + std::to_string(n) + ")", [axis, n](const TermP &p) -> TermP {
        Loop l;
        if (!as_loop(p, l) || l.axis != axis || l.kind != "seq" || l.extent % n == 0) return nullptr;
        return make_loop(axis, (l.extent + n - 1) / n * n, "seq", l.body);
    });
}
// Loop interchange of two directly nested loops over different axes (the sum over k is order free,
// so every interchange of the product's nest is legal; two loops over the same axis are one split
// loop and keep their order).
Strategy<TermP> interchange()
{
    return rule("interchange", [](const TermP &p) -> TermP {
        Loop outer, inner;
        if (!as_loop(p, outer) || !as_loop(outer.body, inner) || outer.axis == inner.axis) return nullptr;
        return make_loop(inner.axis, inner.extent, inner.kind, make_loop(outer.axis, outer.extent, outer.kind, inner.body));
    });
}
// Implementation choices for a sequential loop, the counterpart of rewriting map into mapPar /
// mapSeqUnroll (Section 6.2).  Applicable only where the choice is valid: a wave-parallel loop runs
// over rows or columns of C, never over the reduction; a slab loop is a loop over K; "share" is a
// loop over K whose iterations the waves of a workgroup take side by side (inside a slab; their
// partial sums are added when the K range is done).
Strategy<TermP> mark(const std::string &kind)
{
    return rule("mark(" + kind + ")", [kind](const TermP &p) -> TermP {
        Loop l;
        if (!as_loop(p, l) || l.kind != "seq") return nullptr;
        if (kind == "wave" && l.axis == "K") return nullptr;
        if ((kind == "slab" || kind == "share") && l.axis != "K") return nullptr;
        return make_loop(l.axis, l.extent, kind, l.body);
    });
}
// The matrix instruction: a 32 x 32 x 2 block of multiply-accumulates is one MFMA.
Strategy<TermP> mfma()
{
    return rule("mfma", [](const TermP &p) -> TermP {
        Loop m, n, k;
        if (!as_loop(p, m) || !as_loop(m.body, n) || !as_loop(n.body, k)) return nullptr;
        if (m.axis != "M" || n.axis != "N" || k.axis != "K") return nullptr;
        if (m.extent != 32 || n.extent != 32 || k.extent != 2) return nullptr;
        if (m.kind != "seq" || n.kind != "seq" || k.kind != "seq") return nullptr;
        if (!is_atom(k.body) || k.body->head != "mac") return nullptr;
        return atom("mfma32x32x2");
    });
}

// ---- the image-processing language of Section 5 --------------------------------------------------------
// The binomial filter as the paper writes it, with dot spelled out:
//   (fun img (map2D (fun nbh (reduce add 0 (map mult (zip (join weights2d) (join nbh)))))
//                   (slide2D 3 1 (pad2D 1 img))))
//
// separateDot(w2d, wh, wv), Section 5.2: the dot product of the joined 2-D weights with the joined
// neighbourhood becomes  nbh |> map(dot(wh)) |> dot(wv), written (dot wv (map (dot wh) nbh)).
// Nothing checks that wh and wv separate w2d: that is left to the author of the strategy, as in
// the paper.
Strategy<TermP> separateDot(const TermP &w2d, const TermP &wh, const TermP &wv)
{
    return rule("separateDot", [w2d, wh, wv](const TermP &p) -> TermP {
        if (!is_node(p, "reduce", 3) || !is_atom(p->args[0]) || p->args[0]->head != "add" || !is_atom(p->args[1]) ||
            p->args[1]->head != "0")
            return nullptr;
        const TermP &m = p->args[2];
        if (!is_node(m, "map", 2) || !is_atom(m->args[0]) || m->args[0]->head != "mult") return nullptr;
        const TermP &z = m->args[1];
        if (!is_node(z, "zip", 2) || !is_node(z->args[0], "join", 1) || !is_node(z->args[1], "join", 1)) return nullptr;
        if (!equal(z->args[0]->args[0], w2d)) return nullptr;
        return node("dot", {wv, node("map", {node("dot", {wh}), z->args[1]->args[0]})});
    });
}
// Where the row sums of the separated filter live, the counterpart of Halide's compute_root /
// compute_at for the vertical stage (Section 5.1): (map (dot wh) nbh) under the outer dot becomes
// (stored image ...) -- a whole temporary image -- or (stored line ...) -- the scanline form.
Strategy<TermP> storeRows(const std::string &where)
{
    return rule("storeRows(" + where + ")", [where](const TermP &p) -> TermP {
        if (!is_node(p, "dot", 2) || !is_node(p->args[1], "map", 2) || !is_node(p->args[1]->args[0], "dot", 1)) return nullptr;
        return node("dot", {p->args[0], node("stored", {atom(where), p->args[1]})});
    });
}

// ---- language-specific traversals (Section 3.6) -------------------------------------------------------
Strategy<TermP> child(const std::string &name, const char *head, size_t nargs, size_t index, Strategy<TermP> s,
                      const char *head2 = nullptr, size_t nargs2 = 0, size_t index2 = 0)
{
    const std::string h = head, h2 = head2 ? head2 : "";
    const std::string full = name + "(" + s.name() + ")";
    return Strategy<TermP>(full, [=](const TermP &p) {
        size_t at;
        if (is_node(p, h.c_str(), nargs)) at = index;
        else if (!h2.empty() && is_node(p, h2.c_str(), nargs2)) at = index2;
        else return RewriteResult<TermP>::failure(full);
        RewriteResult<TermP> r = s(p->args[at]);
        if (!r.ok) return r;
        std::vector<TermP> args = p->args;
        args[at] = r.p;
        return RewriteResult<TermP>::success(node(p->head, std::move(args)));
    });
}
// body: the body of a function abstraction, or of a loop
Strategy<TermP> body(Strategy<TermP> s) { return child("body", "fun", 2, 1, s, "loop", 4, 3); }
Strategy<TermP> function(Strategy<TermP> s) { return child("function", "app", 2, 0, s); }
Strategy<TermP> argument(Strategy<TermP> s) { return child("argument", "app", 2, 1, s); }
Strategy<TermP> bodyN(long long n, Strategy<TermP> s)
{
    for (long long i = 0; i < n; ++i) s = body(s);
    return s;
}

// tile(bm, bn) on a nest that starts with a loop over M directly around a loop over N: loop blocking
// of both followed by one interchange, as Section 6.3 builds tiling from split and reorder:
//   M N rest  ->  Mo Mi N rest  ->  Mo Mi No Ni rest  ->  Mo No Mi Ni rest
Strategy<TermP> tile(long long bm, long long bn)
{
    return seq(split("M", bm), seq(bodyN(2, split("N", bn)), body(interchange())));
}

// reorder(p0 p1 ... p_{n-1}): the n outermost perfectly nested loops, numbered 0.. from the outside,
// appear afterwards in the order p0, p1, ...  Built from adjacent interchanges under `body`
// traversals (a selection sort), so it fails exactly where an interchange would be illegal.
Strategy<TermP> reorder(const std::vector<long long> &perm)
{
    std::vector<long long> cur(perm.size());
    for (size_t i = 0; i < cur.size(); ++i) cur[i] = (long long)i;
    Strategy<TermP> s = id<TermP>();
    for (size_t i = 0; i < perm.size(); ++i) {
        size_t j = i;
        while (j < cur.size() && cur[j] != perm[i]) ++j;
        for (; j > i; --j) {                               // bubble the wanted loop outwards
            s = seq(s, bodyN((long long)j - 1, interchange()));
            std::swap(cur[j], cur[j - 1]);
        }
    }
    const size_t n = perm.size();
    return Strategy<TermP>("reorder", [s, n](const TermP &p) {
        TermP t = p;
        for (size_t i = 0; i < n; ++i) {                   // n perfectly nested loops must be there
            Loop l;
            if (!as_loop(t, l)) return RewriteResult<TermP>::failure("reorder");
            t = l.body;
        }
        return s(p);
    });
}

bool ints_from(const TermP &expr, size_t first, std::vector<long long> &out)
{
    for (size_t i = first; i < expr->args.size(); ++i) {
        long long v;
        if (!parse_int(expr->args[i], v)) return false;
        out.push_back(v);
    }
    return true;
}

}  // namespace

Strategy<TermP> compile_strategy(const TermP &e, std::string &err)
{
    typedef Strategy<TermP> S;
    const std::string &h = e->head;
    if (is_atom(e)) {
        if (h == "id") return id<TermP>();
        if (h == "fail") return fail<TermP>();
        if (h == "buildGet") return buildGet();
        if (h == "lenBuild") return lenBuild();
        if (h == "letPartialEval") return letPartialEval();
        if (h == "letApp") return letApp();
        if (h == "funToLet") return funToLet();
        if (h == "interchange") return interchange();
        if (h == "mfma") return mfma();
        err = "unknown strategy '" + h + "'";
        return S();
    }
    // n-ary seq / lChoice fold to the right, as a ; b ; c and a <+ b <+ c read
    if (h == "seq" || h == "lChoice") {
        if (e->args.empty()) { err = h + " needs at least one strategy"; return S(); }
        S acc;
        for (size_t i = e->args.size(); i-- > 0;) {
            S s = compile_strategy(e->args[i], err);
            if (!s) return S();
            acc = acc ? (h == "seq" ? seq(s, acc) : lChoice(s, acc)) : s;
        }
        return acc;
    }
    struct Unary { const char *name; S (*make)(S); };
    static const Unary unary[] = {
        {"try", [](S s) { return try_(s); }},           {"repeat", [](S s) { return repeat(s); }},
        {"all", [](S s) { return all(s); }},            {"one", [](S s) { return one(s); }},
        {"some", [](S s) { return some(s); }},          {"topDown", [](S s) { return topDown(s); }},
        {"bottomUp", [](S s) { return bottomUp(s); }},  {"allTopDown", [](S s) { return allTopDown(s); }},
        {"allBottomUp", [](S s) { return allBottomUp(s); }}, {"tryAll", [](S s) { return tryAll(s); }},
        {"normalize", [](S s) { return normalize(s); }}, {"body", [](S s) { return body(s); }},
        {"function", [](S s) { return function(s); }},  {"argument", [](S s) { return argument(s); }}};
    for (const auto &u : unary) {
        if (h == u.name) {
            if (e->args.size() != 1) { err = h + " takes one strategy"; return S(); }
            S s = compile_strategy(e->args[0], err);
            return s ? u.make(s) : S();
        }
    }
    if (h == "bodyN") {
        long long n;
        if (e->args.size() != 2 || !parse_int(e->args[0], n) || n < 0 || n > 64) { err = "bodyN takes a depth (0..64) and a strategy"; return S(); }
        S s = compile_strategy(e->args[1], err);
        return s ? bodyN(n, s) : S();
    }
    if (h == "split" || h == "cover") {
        long long n;
        if (e->args.size() != 2 || !is_atom(e->args[0]) || !parse_int(e->args[1], n) || n < 1) { err = h + " takes an axis and a positive block size"; return S(); }
        const std::string &axis = e->args[0]->head;
        if (axis != "M" && axis != "N" && axis != "K") { err = h + ": the axis is M, N or K"; return S(); }
        return h == "split" ? split(axis, n) : cover(axis, n);
    }
    if (h == "mark") {
        if (e->args.size() != 1 || !is_atom(e->args[0])) { err = "mark takes a loop kind"; return S(); }
        const std::string &k = e->args[0]->head;
        if (k != "grid" && k != "wave" && k != "unroll" && k != "slab" && k != "share") { err = "mark: the kind is grid, wave, unroll, slab or share"; return S(); }
        return mark(k);
    }
    if (h == "separateDot") {
        if (e->args.size() != 3) { err = "separateDot takes the 2-D weights and the horizontal and vertical weights"; return S(); }
        return separateDot(e->args[0], e->args[1], e->args[2]);
    }
    if (h == "storeRows") {
        if (e->args.size() != 1 || !is_atom(e->args[0]) || (e->args[0]->head != "image" && e->args[0]->head != "line")) {
            err = "storeRows takes image or line";
            return S();
        }
        return storeRows(e->args[0]->head);
    }
    if (h == "tile") {
        std::vector<long long> v;
        if (e->args.size() != 2 || !ints_from(e, 0, v) || v[0] < 1 || v[1] < 1) { err = "tile takes two positive block sizes"; return S(); }
        return tile(v[0], v[1]);
    }
    if (h == "reorder") {
        std::vector<long long> v;
        if (e->args.empty() || e->args.size() > 32 || !ints_from(e, 0, v)) { err = "reorder takes a permutation of 0..n-1"; return S(); }
        std::vector<bool> seen(v.size(), false);
        for (long long x : v) {
            if (x < 0 || x >= (long long)v.size() || seen[(size_t)x]) { err = "reorder takes a permutation of 0..n-1"; return S(); }
            seen[(size_t)x] = true;
        }
        return reorder(v);
    }
    err = "unknown strategy '" + h + "'";
    return S();
}

TermP binomial_filter_program()
{
    std::string err;
    return parse("(fun img (map2D (fun nbh (reduce add 0 (map mult (zip (join weights2d) (join nbh))))) "
                 "(slide2D 3 1 (pad2D 1 img))))", err);
}

namespace {
// counts sub-terms of t (t included) for which pred holds
template <class F> int count_if(const TermP &t, F pred)
{
    int n = pred(t) ? 1 : 0;
    for (const auto &a : t->args) n += count_if(a, pred);
    return n;
}
}  // namespace

int lower_filter(const TermP &program, std::string &err)
{
    const int naive = count_if(program, [](const TermP &t) {
        return is_node(t, "reduce", 3) && is_node(t->args[2], "map", 2) && is_node(t->args[2]->args[1], "zip", 2) &&
               is_node(t->args[2]->args[1]->args[0], "join", 1);
    });
    const int separated = count_if(program, [](const TermP &t) {
        return is_node(t, "dot", 2) && (is_node(t->args[1], "map", 2) || is_node(t->args[1], "stored", 2));
    });
    const int image = count_if(program, [](const TermP &t) { return is_node(t, "stored", 2) && t->args[0]->head == "image"; });
    const int line = count_if(program, [](const TermP &t) { return is_node(t, "stored", 2) && t->args[0]->head == "line"; });
    const int window = count_if(program, [](const TermP &t) { return is_node(t, "slide2D", 3); });
    if (window != 1 || naive + separated != 1) { err = "not a 3x3 filter over one sliding window"; return -1; }
    if (naive == 1) return 0;
    if (image + line != 1) { err = "the separated filter does not say where its row sums are stored"; return -1; }
    return image == 1 ? 1 : 2;
}

TermP product_nest(long long M, long long N, long long K)
{
    return make_loop("M", M, "seq", make_loop("N", N, "seq", make_loop("K", K, "seq", atom("mac"))));
}

bool lower_nest(const TermP &nest, long long M, long long N, long long K, LoweredSchedule &out, std::string &err)
{
    // per axis: product of grid extents, of wave extents, of everything below the grid
    long long grid[3] = {1, 1, 1}, wave[3] = {1, 1, 1}, block[3] = {1, 1, 1}, below_wave[3] = {1, 1, 1};
    long long bk = 0;
    bool seen_non_grid = false, seen_below_wave = false, in_slab = false, seen_slab = false;
    bool k_loop_outside = false, share_without_slab = false;
    TermP t = nest;
    for (int depth = 0;; ++depth) {
        if (depth > 64) { err = "nest too deep"; return false; }
        Loop l;
        if (!as_loop(t, l)) break;
        const int ax = l.axis == "M" ? 0 : (l.axis == "N" ? 1 : 2);
        if (l.kind == "grid") {
            if (seen_non_grid) { err = "a workgroup-parallel loop lies inside a loop of another kind"; return false; }
            if (grid[ax] != 1) { err = "two workgroup-parallel loops over the same axis"; return false; }
            grid[ax] = l.extent;
        } else {
            seen_non_grid = true;
            block[ax] *= l.extent;
            if (l.kind == "share") {
                // waves sharing the reduction: only inside the staged loop, where each takes part of a slab
                // (or with no staged loop at all, when the whole K range is one slab)
                if (!in_slab && k_loop_outside) { err = "a shared loop over the reduction outside the staged loop"; return false; }
                if (wave[2] != 1) { err = "two shared loops"; return false; }
                wave[2] = l.extent;
                if (in_slab) bk *= l.extent;
                else share_without_slab = true;
            } else if (l.kind == "wave") {
                if (seen_below_wave) { err = "a wave-parallel loop lies inside a sequential loop"; return false; }
                if (ax == 2) { err = "a wave-parallel loop over the reduction"; return false; }
                if (wave[ax] != 1) { err = "two wave-parallel loops over the same axis"; return false; }
                wave[ax] = l.extent;
            } else {
                seen_below_wave = true;
                below_wave[ax] *= l.extent;
                if (l.kind == "slab") {
                    if (ax != 2) { err = "a staged loop that is not over K"; return false; }
                    if (seen_slab) { err = "two staged K loops"; return false; }
                    if (share_without_slab) { err = "a staged loop inside a shared loop"; return false; }
                    seen_slab = in_slab = true;
                    bk = 1;
                } else if (l.kind == "seq" || l.kind == "unroll") {
                    if (in_slab && ax == 2) bk *= l.extent;
                    if (!in_slab && ax == 2) k_loop_outside = true;
                } else {
                    err = "unknown loop kind '" + l.kind + "'";
                    return false;
                }
            }
        }
        t = l.body;
    }
    if (!is_atom(t) || t->head != "mfma32x32x2") { err = "the innermost block is not the 32x32x2 matrix instruction"; return false; }
    block[0] *= 32; block[1] *= 32; block[2] *= 2;
    below_wave[0] *= 32; below_wave[1] *= 32;
    bk = seen_slab ? bk * 2 : block[2];      // no staged loop: the whole K range is one slab
    if (grid[0] * block[0] < M || grid[1] * block[1] < N || grid[2] * block[2] < K) { err = "the blocks do not cover the problem"; return false; }
    if ((grid[0] - 1) * block[0] >= M || (grid[1] - 1) * block[1] >= N || (grid[2] > 1 && (grid[2] - 1) * block[2] >= K)) {
        err = "a workgroup-parallel loop has iterations with no work";
        return false;
    }
    out.tiles_m = grid[0]; out.tiles_n = grid[1]; out.split_k = grid[2];
    out.bm = block[0]; out.bn = block[1]; out.k_range = block[2];
    out.bk = bk;
    out.waves_m = wave[0]; out.waves_n = wave[1]; out.waves_k = wave[2];
    out.wave_m = below_wave[0]; out.wave_n = below_wave[1];
    return true;
}

}  // namespace elevate
