// C ABI of the strategy layer (include/elevate.h): text in, text out; the default schedule of the
// product written as a strategy; a scheduled product run on the GPU through the dispatch.
#include "../../include/elevate.h"
#include "../../include/gemm_f32.h"

#include <cstring>
#include <string>
#include <vector>

#include "dispatch.hpp"
#include "elevate.hpp"

using namespace elevate;

namespace {

void put(char *buf, size_t cap, const std::string &s)
{
    if (buf == nullptr || cap == 0) return;
    const size_t n = s.size() < cap - 1 ? s.size() : cap - 1;
    std::memcpy(buf, s.data(), n);
    buf[n] = '\0';
}

// Applies a strategy given as text to a term.  Returns an ELEVATE_* code; `text` is the printed
// result, the failing strategy or the error message.
int apply(const char *strategy, const TermP &program, TermP &result, std::string &text, Trace &trace)
{
    std::string err;
    const TermP expr = parse(strategy, err);
    if (!expr) { text = "strategy: " + err; return ELEVATE_EPARSE; }
    const Strategy<TermP> s = compile_strategy(expr, err);
    if (!s) { text = "strategy: " + err; return ELEVATE_EPARSE; }
    current_trace() = &trace;
    const RewriteResult<TermP> r = s(program);
    current_trace() = nullptr;
    if (trace.exhausted) { text = "step limit reached"; return ELEVATE_ELIMIT; }
    if (!r.ok) { text = r.failed; return ELEVATE_FAILED; }
    result = r.p;
    text = print(r.p);
    return ELEVATE_OK;
}

struct NestLoop { char axis; long long extent; const char *kind; };   // kind: the role the loop gets

// The schedule of one of the library's kernels as a strategy over the plain nest M N K:
// cover the ragged edges, block every axis (workgroup tile, wave tile, 32x32x2 instruction; K range,
// slab, instruction), reorder into grid / waves / slab / steps / register block / instruction, give
// every loop its implementation, and turn the innermost block into the matrix instruction.
std::string default_strategy(long long M, long long N, long long K, const gemmf32_host::TileChoice &c)
{
    const long long wave_m = c.bm / c.waves_m, wave_n = c.bn / c.waves_n;
    const long long k_range = c.split > 1 ? ((K + c.split - 1) / c.split + c.bk - 1) / c.bk * c.bk
                                          : (K + c.bk - 1) / c.bk * c.bk;
    std::vector<NestLoop> nest = {{'M', M, "seq"}, {'N', N, "seq"}, {'K', K, "seq"}};
    std::string s = "(seq";
    auto emit = [&](const std::string &step) { s += " " + step; };
    auto pos_of = [&](char axis) {                                    // innermost loop of the axis
        size_t p = nest.size();
        for (size_t i = 0; i < nest.size(); ++i)
            if (nest[i].axis == axis) p = i;
        return p;
    };
    auto cover_axis = [&](char axis, long long n) {
        const size_t p = pos_of(axis);
        if (nest[p].extent % n != 0) {
            emit("(bodyN " + std::to_string(p) + " (cover " + std::string(1, axis) + " " + std::to_string(n) + "))");
            nest[p].extent = (nest[p].extent + n - 1) / n * n;
        }
    };
    // splits the innermost loop of `axis` by n; the outer part gets role `outer`
    auto split_axis = [&](char axis, long long n, const char *outer) {
        const size_t p = pos_of(axis);
        if (nest[p].extent <= n) return;
        emit("(bodyN " + std::to_string(p) + " (split " + std::string(1, axis) + " " + std::to_string(n) + "))");
        const long long e = nest[p].extent;
        nest[p] = NestLoop{axis, (e + n - 1) / n, outer};
        nest.insert(nest.begin() + (long)p + 1, NestLoop{axis, n, "seq"});
    };
    cover_axis('M', c.bm);
    cover_axis('N', c.bn);
    cover_axis('K', k_range);
    split_axis('M', c.bm, "grid");
    split_axis('M', wave_m, "wave");
    split_axis('M', 32, "unroll");
    split_axis('N', c.bn, "grid");
    split_axis('N', wave_n, "wave");
    split_axis('N', 32, "unroll");
    split_axis('K', k_range, "grid");
    split_axis('K', c.bk, "slab");
    if (c.waves_k > 1) split_axis('K', c.bk / c.waves_k, "kwave");     // the waves share every slab
    split_axis('K', 2, "step");
    // wanted order: grid loops, wave loops, slab, k steps, register block, the instruction's M N K
    static const char *order[] = {"grid", "wave", "slab", "kwave", "step", "unroll", "seq"};
    std::vector<size_t> perm;
    for (const char *role : order)
        for (char axis : {'M', 'N', 'K'})
            for (size_t i = 0; i < nest.size(); ++i)
                if (nest[i].axis == axis && std::strcmp(nest[i].kind, role) == 0) perm.push_back(i);
    bool identity = true;
    for (size_t i = 0; i < perm.size(); ++i) identity = identity && perm[i] == i;
    if (!identity) {
        std::string r = "(reorder";
        for (size_t i : perm) r += " " + std::to_string(i);
        emit(r + ")");
    }
    for (size_t i = 0; i < perm.size(); ++i) {
        const char *role = nest[perm[i]].kind;
        if (std::strcmp(role, "seq") != 0 && std::strcmp(role, "step") != 0)
            emit("(bodyN " + std::to_string(i) + " (mark " + (std::strcmp(role, "kwave") == 0 ? "share" : role) + "))");
    }
    emit("(topDown mfma)");
    return s + ")";
}

// reads M, N, K off a plain product nest (loop M m seq (loop N n seq (loop K k seq mac)))
bool plain_extents(const TermP &p, long long &M, long long &N, long long &K)
{
    const TermP *t = &p;
    long long *out[3] = {&M, &N, &K};
    const char *axes[3] = {"M", "N", "K"};
    for (int i = 0; i < 3; ++i) {
        if (!is_node(*t, "loop", 4) || !is_atom((*t)->args[0]) || (*t)->args[0]->head != axes[i] || !is_atom((*t)->args[1])) return false;
        *out[i] = std::atoll((*t)->args[1]->head.c_str());
        t = &(*t)->args[3];
    }
    return true;
}

}  // namespace

namespace gemmf32_host {

// The dispatch as a strategy: (lChoice c0 c1 ...), one candidate per tile shape, each
//     c = (seq admissible(tile) cheapest(tile) schedule(tile, split))
// where the first two are guards (they leave the nest as it is, or fail) and the third is the schedule of
// default_strategy for that tile.  Applied to the plain nest of the product; the result is lowered.
bool dispatch_by_strategy(const ShapeQuery &q, const TileChoice &cheapest, TileChoice &lowered)
{
    Strategy<TermP> dispatch = fail<TermP>();
    for (int tile = tile_count() - 1; tile >= 0; --tile) {
        const TileChoice shape = tile_shape(tile);
        const Strategy<TermP> may_compete("admissible", [tile, q](const TermP &p) {
            long long M, N, K;
            if (!plain_extents(p, M, N, K)) return RewriteResult<TermP>::failure("admissible");
            ShapeQuery here = q;
            here.M = M; here.N = N; here.K = K;
            return admissible_tile(tile, here) ? RewriteResult<TermP>::success(p) : RewriteResult<TermP>::failure("admissible");
        });
        const Strategy<TermP> is_cheapest("cheapest", [shape, cheapest](const TermP &p) {
            const bool same = shape.bm == cheapest.bm && shape.bn == cheapest.bn && shape.bk == cheapest.bk &&
                              shape.waves_m == cheapest.waves_m && shape.waves_n == cheapest.waves_n &&
                              shape.waves_k == cheapest.waves_k;
            return same ? RewriteResult<TermP>::success(p) : RewriteResult<TermP>::failure("cheapest");
        });
        const Strategy<TermP> schedule("schedule", [shape, cheapest](const TermP &p) {
            long long M, N, K;
            if (!plain_extents(p, M, N, K)) return RewriteResult<TermP>::failure("schedule");
            TileChoice c = shape;
            c.split = cheapest.split;
            std::string err;
            const TermP expr = parse(default_strategy(M, N, K, c), err);
            if (!expr) return RewriteResult<TermP>::failure("schedule");
            const Strategy<TermP> s = compile_strategy(expr, err);
            if (!s) return RewriteResult<TermP>::failure("schedule");
            return s(p);
        });
        dispatch = lChoice(seq(may_compete, seq(is_cheapest, schedule)), dispatch);
    }
    const RewriteResult<TermP> r = dispatch(product_nest(q.M, q.N, q.K));
    if (!r.ok) return false;
    LoweredSchedule ls;
    std::string err;
    if (!lower_nest(r.p, q.M, q.N, q.K, ls, err)) return false;
    const long long big = 2147483647LL;
    if (ls.bm > big || ls.bn > big || ls.bk > big || ls.waves_m > big || ls.waves_n > big || ls.waves_k > big || ls.split_k > big) return false;
    lowered = TileChoice{(int)ls.bm, (int)ls.bn, (int)ls.bk, (int)ls.waves_m, (int)ls.waves_n, (int)ls.waves_k, (int)ls.split_k};
    return true;
}

}  // namespace gemmf32_host

extern "C" {

void elevate_dispatch_stats(int64_t *applied, int64_t *failed)
{
    long long a = 0, f = 0;
    gemmf32_host::strategy_dispatch_stats(&a, &f);
    if (applied) *applied = a;
    if (failed) *failed = f;
}

int elevate_rewrite(const char *strategy, const char *program, char *out, size_t out_cap, int *steps, char *trace_buf,
                    size_t trace_cap)
{
    if (steps) *steps = 0;
    put(out, out_cap, "");
    put(trace_buf, trace_cap, "");
    if (strategy == nullptr || program == nullptr) return ELEVATE_ENULL;
    std::string err;
    const TermP p = parse(program, err);
    if (!p) {
        put(out, out_cap, "program: " + err);
        return ELEVATE_EPARSE;
    }
    Trace trace;
    TermP result;
    std::string text;
    const int rc = apply(strategy, p, result, text, trace);
    put(out, out_cap, text);
    if (steps) *steps = (int)trace.steps.size();
    if (trace_buf != nullptr && trace_cap > 0) {
        std::string t;
        for (const auto &st : trace.steps) t += st.rule + ": " + st.before + " => " + st.after + "\n";
        put(trace_buf, trace_cap, t);
    }
    return rc;
}

int elevate_alpha_equal(const char *a, const char *b)
{
    if (a == nullptr || b == nullptr) return ELEVATE_ENULL;
    std::string err;
    const TermP ta = parse(a, err), tb = parse(b, err);
    if (!ta || !tb) return ELEVATE_EPARSE;
    return alpha_equal(ta, tb) ? 1 : 0;
}

int elevate_schedule_gemm(int64_t M, int64_t N, int64_t K, const char *strategy, gemmf32_schedule *out, char *nest_buf,
                          size_t nest_cap)
{
    put(nest_buf, nest_cap, "");
    if (strategy == nullptr || out == nullptr) return ELEVATE_ENULL;
    std::memset(out, 0, sizeof(*out));
    if (M < 1 || N < 1 || K < 1 || M > 2147483647LL || N > 2147483647LL || K > 2147483647LL) {
        put(nest_buf, nest_cap, "dimensions must be between 1 and 2^31-1");
        return ELEVATE_EPARSE;
    }
    Trace trace;
    TermP nest;
    std::string text;
    const int rc = apply(strategy, product_nest(M, N, K), nest, text, trace);
    put(nest_buf, nest_cap, text);
    if (rc != ELEVATE_OK) return rc;
    LoweredSchedule ls;
    std::string err;
    if (!lower_nest(nest, M, N, K, ls, err)) {
        put(nest_buf, nest_cap, err);
        return ELEVATE_ELOWER;
    }
    const long long big = 2147483647LL;
    if (ls.bm > big || ls.bn > big || ls.bk > big || ls.waves_m > big || ls.waves_n > big || ls.waves_k > big || ls.split_k > big) {
        put(nest_buf, nest_cap, "block sizes out of range");
        return ELEVATE_ELOWER;
    }
    out->bm = (int32_t)ls.bm; out->bn = (int32_t)ls.bn; out->bk = (int32_t)ls.bk;
    out->waves_m = (int32_t)ls.waves_m; out->waves_n = (int32_t)ls.waves_n; out->waves_k = (int32_t)ls.waves_k;
    out->wave_m = (int32_t)(ls.wave_m > big ? big : ls.wave_m);
    out->wave_n = (int32_t)(ls.wave_n > big ? big : ls.wave_n);
    out->split_k = (int32_t)ls.split_k;
    out->tiles_m = ls.tiles_m; out->tiles_n = ls.tiles_n;
    out->k_range = ls.k_range;
    const bool built = gemmf32_host::has_kernel(out->bm, out->bn, out->bk, out->waves_m, out->waves_n, out->waves_k) &&
                       (int64_t)out->wave_m * out->waves_m == out->bm && (int64_t)out->wave_n * out->waves_n == out->bn;
    return built ? ELEVATE_OK : ELEVATE_ENOKERNEL;
}

int elevate_schedule_filter(const char *strategy, int *form, char *program_buf, size_t program_cap)
{
    put(program_buf, program_cap, "");
    if (strategy == nullptr || form == nullptr) return ELEVATE_ENULL;
    *form = -1;
    Trace trace;
    TermP program;
    std::string text;
    const int rc = apply(strategy, binomial_filter_program(), program, text, trace);
    put(program_buf, program_cap, text);
    if (rc != ELEVATE_OK) return rc;
    std::string err;
    const int f = lower_filter(program, err);
    if (f < 0) {
        put(program_buf, program_cap, err);
        return ELEVATE_ELOWER;
    }
    *form = f;
    return ELEVATE_OK;
}

int elevate_default_strategy(int64_t M, int64_t N, int64_t K, char *strategy, size_t cap)
{
    put(strategy, cap, "");
    if (strategy == nullptr) return ELEVATE_ENULL;
    if (M < 1 || N < 1 || K < 1 || M > 2147483647LL || N > 2147483647LL || K > 2147483647LL) return ELEVATE_EPARSE;
    const std::string s = default_strategy(M, N, K, gemmf32_host::choose(M, N, K));
    if (s.size() + 1 > cap) return ELEVATE_EPARSE;
    put(strategy, cap, s);
    return ELEVATE_OK;
}

int gemm_f32_scheduled(const gemmf32_schedule *s, int64_t M, int64_t N, int64_t K, const float *A, int64_t lda,
                       const float *B, int64_t ldb, float *C, int64_t ldc, int transB)
{
    if (s == nullptr) return GEMMF32_ENULL;
    if (!gemmf32_host::has_kernel(s->bm, s->bn, s->bk, s->waves_m, s->waves_n, s->waves_k)) return GEMMF32_EINVAL;
    if (s->split_k < 1) return GEMMF32_EINVAL;
    if (M > 0 && N > 0 && K > 0) {
        // the schedule must be one for this problem: its blocks cover it with no idle workgroup
        const int64_t tiles_m = (M + s->bm - 1) / s->bm, tiles_n = (N + s->bn - 1) / s->bn;
        if (s->tiles_m != tiles_m || s->tiles_n != tiles_n) return GEMMF32_EINVAL;
        const int64_t per = (K + s->split_k - 1) / s->split_k;
        const int64_t k_range = (per + s->bk - 1) / s->bk * s->bk;
        if (s->k_range != k_range || (K + k_range - 1) / k_range != s->split_k) return GEMMF32_EINVAL;
    }
    return gemmf32_host::run_forced(s->bm, s->bn, s->bk, s->split_k, M, N, K, A, lda, B, ldb, C, ldc, transB);
}

}  // extern "C"
