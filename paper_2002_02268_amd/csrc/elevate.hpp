// A small strategy language for program rewriting, after Section 3 of the paper (ELEVATE):
// strategies are functions from a program to success-with-a-new-program or failure-naming-the-
// strategy-that-failed; rewrite rules are strategies; combinators (seq, lChoice, try, repeat),
// one-level traversals (all, one, some) and whole-term traversals (topDown, bottomUp, allTopDown,
// allBottomUp, tryAll, normalize) are built from each other exactly as Section 3.4-3.8 defines
// them.  Host code only; nothing here touches the GPU.
//
// Programs are terms: an atom (a name or a number) or a head with arguments, written as
// s-expressions.  Two small languages are expressed in them (see elevate.cpp): the functional
// array language of Section 4 (build / get / length / let / fun / app) and a perfect loop nest
// over the axes M, N, K of the matrix product that stands where Section 6 uses RISE.
#pragma once

#include <functional>
#include <memory>
#include <string>
#include <utility>
#include <vector>

namespace elevate {

// ---- terms ---------------------------------------------------------------------------------------
struct Term;
typedef std::shared_ptr<const Term> TermP;
struct Term {
    std::string head;            // atom text, or the head symbol of a compound term
    std::vector<TermP> args;     // empty for an atom
    bool compound;               // "(f)" is compound with no arguments, "f" is an atom
};

inline TermP atom(const std::string &s)
{
    return std::make_shared<const Term>(Term{s, {}, false});
}
inline TermP node(const std::string &head, std::vector<TermP> args)
{
    return std::make_shared<const Term>(Term{head, std::move(args), true});
}
inline bool is_atom(const TermP &t) { return !t->compound; }
inline bool is_node(const TermP &t, const char *head, size_t nargs)
{
    return t->compound && t->head == head && t->args.size() == nargs;
}

bool equal(const TermP &a, const TermP &b);
std::string print(const TermP &t);
// Parses one s-expression; on error returns nullptr and sets err.
TermP parse(const std::string &text, std::string &err);

// ---- rewrite results and strategies (Section 3.2) ------------------------------------------------
template <class P> struct RewriteResult {
    bool ok;
    P p;                     // the rewritten program when ok
    std::string failed;      // the strategy that was unsuccessful when !ok
    static RewriteResult success(P q) { return RewriteResult{true, std::move(q), std::string()}; }
    static RewriteResult failure(std::string who) { return RewriteResult{false, P(), std::move(who)}; }
};

// (name and function live behind a shared pointer: combinators capture their arguments by value, and a
// chain of n of them would otherwise copy closures of closures n^2 / 2 times)
template <class P> class Strategy {
public:
    typedef std::function<RewriteResult<P>(const P &)> Fn;
    Strategy() {}
    Strategy(std::string name, Fn fn) : impl_(std::make_shared<const Impl>(Impl{std::move(name), std::move(fn)})) {}
    RewriteResult<P> operator()(const P &p) const { return impl_->fn(p); }
    const std::string &name() const
    {
        static const std::string none;
        return impl_ ? impl_->name : none;
    }
    explicit operator bool() const { return impl_ && (bool)impl_->fn; }

private:
    struct Impl {
        std::string name;
        Fn fn;
    };
    std::shared_ptr<const Impl> impl_;
};

// Every successful application of a rewrite rule is recorded here (rule name, the sub-term it
// matched, what it became), in order.  A step limit turns a non-terminating strategy (Section 3.8
// leaves termination to the author of the strategy) into an error instead of a hang.
struct Trace {
    struct Step { std::string rule, before, after; };
    std::vector<Step> steps;
    size_t limit = 100000;
    bool exhausted = false;
};
Trace *&current_trace();   // thread-local; null: nothing recorded, no limit

// A rewrite rule: a strategy that matches the root of the program it is given (Section 3.3).
// `fn` returns the rewritten term or nullptr when the rule does not apply.
Strategy<TermP> rule(const std::string &name, std::function<TermP(const TermP &)> fn);

template <class P> Strategy<P> id()
{
    return Strategy<P>("id", [](const P &p) { return RewriteResult<P>::success(p); });
}
template <class P> Strategy<P> fail()
{
    return Strategy<P>("fail", [](const P &) { return RewriteResult<P>::failure("fail"); });
}

// ---- combinators (Section 3.4) -------------------------------------------------------------------
// seq: the second strategy is applied to the result of the first; fails if either fails.
template <class P> Strategy<P> seq(Strategy<P> fs, Strategy<P> ss)
{
    return Strategy<P>("(" + fs.name() + " ; " + ss.name() + ")", [fs, ss](const P &p) {
        RewriteResult<P> r = fs(p);
        return r.ok ? ss(r.p) : r;
    });
}
// lChoice: the second strategy is applied (to the original program) only if the first failed.
template <class P> Strategy<P> lChoice(Strategy<P> fs, Strategy<P> ss)
{
    return Strategy<P>("(" + fs.name() + " <+ " + ss.name() + ")", [fs, ss](const P &p) {
        RewriteResult<P> r = fs(p);
        return r.ok ? r : ss(p);
    });
}
// try: the strategy, or the identity if it fails; never fails.
template <class P> Strategy<P> try_(Strategy<P> s) { return lChoice(s, id<P>()); }
// repeat: the strategy until it is no longer applicable:  repeat(s) = try(s ; repeat(s)).
// The recursion of the definition is unrolled into a loop (same result, no stack growth per step).
template <class P> Strategy<P> repeat(Strategy<P> s)
{
    return Strategy<P>("repeat(" + s.name() + ")", [s](const P &p) {
        P cur = p;
        for (;;) {
            RewriteResult<P> r = s(cur);
            if (!r.ok) return RewriteResult<P>::success(cur);
            cur = r.p;
        }
    });
}

// ---- one-level traversals (Section 3.5): a type class over the program type -----------------------
template <class P> struct Traversable;   // children(p), rebuild(p, children)

template <> struct Traversable<TermP> {
    static std::vector<TermP> children(const TermP &p) { return p->args; }
    static TermP rebuild(const TermP &p, std::vector<TermP> kids)
    {
        return p->compound ? node(p->head, std::move(kids)) : p;
    }
};

// all: the strategy applied to every sub-expression; fails if it fails on one of them.
template <class P> Strategy<P> all(Strategy<P> s)
{
    return Strategy<P>("all(" + s.name() + ")", [s](const P &p) {
        std::vector<P> kids = Traversable<P>::children(p);
        for (auto &k : kids) {
            RewriteResult<P> r = s(k);
            if (!r.ok) return r;
            k = r.p;
        }
        return RewriteResult<P>::success(Traversable<P>::rebuild(p, std::move(kids)));
    });
}
// one: the strategy applied to exactly one sub-expression, the leftmost on which it succeeds
// (the choice the paper leaves to the implementation is made deterministic here).
template <class P> Strategy<P> one(Strategy<P> s)
{
    return Strategy<P>("one(" + s.name() + ")", [s](const P &p) {
        std::vector<P> kids = Traversable<P>::children(p);
        for (auto &k : kids) {
            RewriteResult<P> r = s(k);
            if (r.ok) {
                k = r.p;
                return RewriteResult<P>::success(Traversable<P>::rebuild(p, std::move(kids)));
            }
        }
        return RewriteResult<P>::failure("one(" + s.name() + ")");
    });
}
// some: the strategy applied to every sub-expression on which it succeeds; fails if there is none.
template <class P> Strategy<P> some(Strategy<P> s)
{
    return Strategy<P>("some(" + s.name() + ")", [s](const P &p) {
        std::vector<P> kids = Traversable<P>::children(p);
        bool any = false;
        for (auto &k : kids) {
            RewriteResult<P> r = s(k);
            if (r.ok) {
                k = r.p;
                any = true;
            }
        }
        if (!any) return RewriteResult<P>::failure("some(" + s.name() + ")");
        return RewriteResult<P>::success(Traversable<P>::rebuild(p, std::move(kids)));
    });
}

// ---- whole-expression traversals (Section 3.7) and normalisation (Section 3.8) ---------------------
template <class P> Strategy<P> topDown(Strategy<P> s)
{
    return Strategy<P>("topDown(" + s.name() + ")", [s](const P &p) { return lChoice(s, one(topDown(s)))(p); });
}
template <class P> Strategy<P> bottomUp(Strategy<P> s)
{
    return Strategy<P>("bottomUp(" + s.name() + ")", [s](const P &p) { return lChoice(one(bottomUp(s)), s)(p); });
}
template <class P> Strategy<P> allTopDown(Strategy<P> s)
{
    return Strategy<P>("allTopDown(" + s.name() + ")", [s](const P &p) { return seq(s, all(allTopDown(s)))(p); });
}
template <class P> Strategy<P> allBottomUp(Strategy<P> s)
{
    return Strategy<P>("allBottomUp(" + s.name() + ")", [s](const P &p) { return seq(all(allBottomUp(s)), s)(p); });
}
template <class P> Strategy<P> tryAll(Strategy<P> s)
{
    return Strategy<P>("tryAll(" + s.name() + ")",
                       [s](const P &p) { return seq(all(tryAll(try_(s))), try_(s))(p); });
}
template <class P> Strategy<P> normalize(Strategy<P> s) { return repeat(topDown(s)); }

// ---- the two term languages and the strategy expressions over them (elevate.cpp) -------------------
// Compiles a strategy written as an s-expression, e.g.
//   (normalize (lChoice buildGet lenBuild letPartialEval letApp funToLet))
//   (seq (tile 256 256) (bodyN 4 (split K 16)))
// into a strategy over terms.  Returns an empty strategy and sets err on an unknown name or a
// malformed argument list.
Strategy<TermP> compile_strategy(const TermP &expr, std::string &err);

// Capture-avoiding substitution e[x := v] and alpha-equivalence for the functional language.
TermP substitute(const TermP &e, const std::string &x, const TermP &v);
bool alpha_equal(const TermP &a, const TermP &b);

// The 3x3 binomial filter of Section 5 in its naive form, and what a rewritten form says about the
// kernel that runs it: 0 naive (nine taps per pixel), 1 separated with the row sums in a temporary
// image, 2 scanline (row sums kept per line); -1 (and err) if the program is none of these.
TermP binomial_filter_program();
int lower_filter(const TermP &program, std::string &err);

// The loop nest of the plain product: (loop M m seq (loop N n seq (loop K k seq mac))).
TermP product_nest(long long M, long long N, long long K);

// What a scheduled nest says about the kernel that runs it.
struct LoweredSchedule {
    long long tiles_m, tiles_n, split_k;     // extents of the workgroup-parallel loops
    long long bm, bn, k_range;               // per-workgroup block: rows, columns, length of its K range
    long long bk;                            // K extent staged through LDS per slab
    long long waves_m, waves_n;              // waves per workgroup along M and N
    long long waves_k;                       // waves that split every K slab between them (1: none)
    long long wave_m, wave_n;                // rows / columns of C per wave (register block x MFMA block)
};
// Reads the kernel configuration off a scheduled nest; false (and err) if the nest is not a
// schedule a kernel can execute (parallel loops below sequential ones, no staged K loop, no MFMA
// leaf, blocks that do not cover the problem, ...).
bool lower_nest(const TermP &nest, long long M, long long N, long long K, LoweredSchedule &out, std::string &err);

}  // namespace elevate
