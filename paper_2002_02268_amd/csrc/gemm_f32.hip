// C-ABI entry points and dispatch for the fp32 matrix product on gfx950.
// Argument checks, choice of tile variant from the shape, launch on the configured stream.
#include "../../include/gemm_f32.h"
#include "../../include/gemm_f32_testing.h"

#include <type_traits>

#include "dispatch.hpp"
#include "gemm_launch.hpp"

#include <algorithm>
#include <atomic>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <unordered_map>
#include <vector>

using namespace gemmf32;

// Scratch of gemm_f32_noalloc (see there): a fixed array in the code object, one copy per device.
constexpr size_t kScratchBytes = 32u << 20;
static __device__ __align__(256) float scratch[kScratchBytes / sizeof(float)];

namespace {

// Each host thread has its own current stream, so threads that drive different streams do not
// disturb each other.
thread_local hipStream_t g_stream = nullptr;
thread_local int g_last_hip_error = 0;
#ifdef GEMMF32_TIMELINE
unsigned long long *g_timeline_stamps = nullptr;   // measurement build only (see the kernel header)
#endif

constexpr int64_t kMaxDim = 2147483647LL;
constexpr int64_t kMaxElems = 1LL << 40;

int fail_hip(hipError_t e)
{
    g_last_hip_error = (int)e;
    return GEMMF32_ELAUNCH;
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace

using namespace gemmf32_host;

namespace gemmf32_host {
hipStream_t current_stream() { return g_stream; }
int record_hip_error(hipError_t e) { return fail_hip(e); }
extern template int launch_tile<B_NN, A_MK>(int, const KArgs &);
extern template int launch_tile<B_NT, A_MK>(int, const KArgs &);
extern template int launch_tile<B_PACKED, A_MK>(int, const KArgs &);
extern template int launch_tile<B_NN, A_KM>(int, const KArgs &);
extern template int launch_tile<B_NT, A_KM>(int, const KArgs &);
}  // namespace gemmf32_host

namespace {

int launch_variant(int bmode, int amode, int tile, const KArgs &a)
{
    if (amode == A_KM) {
        if (bmode == B_NN) return launch_tile<B_NN, A_KM>(tile, a);
        if (bmode == B_NT) return launch_tile<B_NT, A_KM>(tile, a);
        return GEMMF32_EINVAL;          // no packed B with A stored K x M
    }
    switch (bmode) {
    case B_NN: return launch_tile<B_NN, A_MK>(tile, a);
    case B_NT: return launch_tile<B_NT, A_MK>(tile, a);
    default: return launch_tile<B_PACKED, A_MK>(tile, a);
    }
}

int64_t cdiv(int64_t a, int64_t b) { return (a + b - 1) / b; }

template <int BMODE> int launch_batched64_mode(const BatchArgs &a)
{
    constexpr int SB = (BMODE == B_NT) ? 68 : 64;
    constexpr int lds_bytes = 2 * (64 * 68 + 64 * SB) * 4;
    static std::atomic<uint64_t> lds_limit_set{0};
    auto kern = batched64_kernel<BMODE>;
    const int rc = ensure_lds_limit(reinterpret_cast<const void *>(kern), lds_bytes, lds_limit_set);
    if (rc != GEMMF32_OK) return rc;
    // two workgroups per compute unit (what the LDS holds); more residency does not raise the
    // achieved bandwidth, which already equals that of a plain device copy
    const int grid = a.batch < 512 ? a.batch : 512;
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(256), lds_bytes, g_stream, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail_hip(e);
    return GEMMF32_OK;
}

int launch_batched64(int64_t batch, const float *A, int64_t lda, int64_t sA, const float *B, int64_t ldb,
                     int64_t sB, float *C, int64_t ldc, int64_t sC, int transB)
{
    BatchArgs a;
    a.A = A; a.B = B; a.C = C;
    a.lda = lda; a.ldb = ldb; a.ldc = ldc;
    a.sA = sA; a.sB = sB; a.sC = sC;
    a.batch = (int)batch;
    return transB ? launch_batched64_mode<B_NT>(a) : launch_batched64_mode<B_NN>(a);
}

// Tile and split choice.  Workgroups spread over 256 compute units, so a launch costs
// ceil(workgroups / 256) rounds of one tile each.  A tile over a K range of length k costs
// 2*BM*BN*(k + overhead) flops at the fraction of one compute unit's MFMA peak (0.6144 Tflop/s)
// that the variant sustains (VariantModel below).  Splitting K into S ranges multiplies the workgroups by S and adds a
// second pass that sums S partial products.  The cheapest (variant, S) wins: big tiles when they
// fill the chip evenly, smaller ones when the last round would be mostly empty, a K split when
// the output alone cannot occupy the chip.
constexpr double kCuFlopsPerUs = 157.3e6 / 256.0;
constexpr int64_t kMaxWorkspaceBytes = 256LL << 20;

struct Choice { int tile; int split; int strip; };   // strip: last columns of C left to the strip workgroups (0: none)

// What each variant sustains, fitted to measurements: the fraction of a compute unit's MFMA peak when
// the launch is a single round of workgroups (`single`) and when several workgroups per compute unit
// follow or overlap each other (`multi`: the small tiles hide their load latency behind a co-resident
// neighbour), and the fixed cost of a tile (first-slab latency, epilogue) in both regimes,
// expressed as extra columns of K.
struct VariantModel { int id; double single, multi, overhead_single, overhead_multi; };
const VariantModel kCandidates[] = {
    {T256, 0.975, 0.976, 63, 53},      {T256x128, 0.956, 0.962, 71, 27},  {T128x256, 0.957, 0.965, 72, 26},
    {T128, 0.967, 0.976, 103, 40},     {T64x128, 0.950, 0.972, 153, 64},  {T128x64, 0.958, 0.973, 159, 69},
    {TB64, 0.947, 0.963, 259, 110},    {T64, 0.904, 0.954, 213, 90},
    {T128x32, 0.898, 0.933, 223, 294}, {T32x128, 0.895, 0.797, 223, 110},
    {TQ32, 0.715, 0.837, 510, 241},    {TQ64x32, 0.874, 0.900, 429, 188}, {TQ32x64, 0.857, 0.919, 440, 245}};
// (Of the two orientations of the 128 x 64 tile the one with the longer rows of B comes first and so wins a tie:
// measured, it is 1-2 % ahead on outputs of five hundred tiles or more, 4352 x 4352 x 4096 1049 against 1068 us,
// 6144^3 3162 against 3224, and level with the other below that.)
const VariantModel &variant_model(int tile)
{
    for (const auto &c : kCandidates)
        if (c.id == tile) return c;
    return kCandidates[6];
}
// modelled microseconds of one tile of the variant over a K range of length k
double tile_us(const VariantModel &v, int bm, int bn, double k, bool multi)
{
    return 2.0 * bm * bn * (k + (multi ? v.overhead_multi : v.overhead_single)) /
           (kCuFlopsPerUs * (multi ? v.multi : v.single));
}

// Split of the last, partly filled round: `tail` tiles cut into `pieces` K ranges of `piece_k` columns
// each (pieces <= 1: no split).  benefit_us: modelled time saved against running the tail as a round
// of whole tiles, the second pass already charged.
// quad: instead, every tail tile is cut into its 32 x 32 blocks (`pieces` of them), each computed by a
// whole workgroup whose waves share the slabs along k: a quarter of a tile's time per block, and no
// second pass.  Better than K ranges when K is short (the second pass costs its launch whatever K is).
// Test hooks (gemm_f32_set_test_hooks): process-wide, all off in production.  The environment is never read.
struct Hooks {
    bool no_tail_split, no_quad, no_kshare, no_thin, force_thin;
    int force_tile, force_split;       // -1: not forced
    bool no_strip;
    int strip_wait;                    // -1: the library's own
    bool force_strip;
    int strip_rows;                    // 0: the library's own
};
struct HookState {
    std::atomic<int> force_tile{-1}, force_split{-1};
    std::atomic<int> no_tail_split{0}, no_quad{0}, no_kshare{0}, no_thin{0}, force_thin{0}, no_strip{0}, strip_wait{0}, force_strip{0}, strip_rows{0};
} g_hooks;
Hooks read_hooks()
{
    const auto get = [](const std::atomic<int> &a) { return a.load(std::memory_order_relaxed); };
    return Hooks{get(g_hooks.no_tail_split) != 0, get(g_hooks.no_quad) != 0, get(g_hooks.no_kshare) != 0,
                 get(g_hooks.no_thin) != 0,       get(g_hooks.force_thin) != 0, get(g_hooks.force_tile),
                 get(g_hooks.force_split),        get(g_hooks.no_strip) != 0,   get(g_hooks.strip_wait) - 1,
                 get(g_hooks.force_strip) != 0,   get(g_hooks.strip_rows)};
}

// Columns of C left to the strip workgroups (kernel header, KArgs): when N is at most kStripMax columns more
// than whole tiles, one product, no K ranges, A stored M x K, B not packed, a tile of four waves that each own
// blocks.  0: no strip (the last tile column is an edge tile).
int strip_cols(const Hooks &hooks, int tile, int64_t batch, int64_t N, int bmode, int amode)
{
    const TileShape &sh = kShapes[tile];
    if (hooks.no_strip || batch != 1 || amode != A_MK || bmode == B_PACKED) return 0;
    if (sh.waves_k != 1 || sh.waves_m * sh.waves_n != 4) return 0;
    const int64_t rest = N % sh.bn;
    return (N >= sh.bn && rest >= 1 && rest <= kStripMax) ? (int)rest : 0;
}

struct TailSplit { int64_t tail; int64_t pieces; int64_t piece_k; double benefit_us; bool quad; };

TailSplit plan_tail_split(const Hooks &hooks, int tile, int64_t batch, int64_t tiles, int64_t K)
{
    const VariantModel &vm = variant_model(tile);
    const int bm = kShapes[tile].bm, bn = kShapes[tile].bn, bk = kShapes[tile].bk;
    TailSplit t = {tiles % 256, 1, 0, 0.0, false};
    if (batch != 1 || tiles <= 256 || t.tail == 0 || t.tail > 128 || hooks.no_tail_split) return t;
    const int64_t units = cdiv(K, bk);
    if (units < 2) return t;                             // nothing to cut (K = 0 included)
    int64_t S = 256 / t.tail;
    if (S > 8) S = 8;     // shorter pieces than an eighth of K cost more in the second pass than they save
    if (S > units) S = units;
    const int64_t units_per_piece = cdiv(units, S);
    S = cdiv(units, units_per_piece);                    // no empty pieces
    const double t_full = tile_us(vm, bm, bn, (double)K, true);
    // 32 x 32 blocks: measured, a round of them adds 5 us + 1.8 ns per column of K to the launch (they
    // start on compute units whose whole tiles ended early); in proportion if there are more than 256
    double quad_benefit = 0.0;
    const int64_t subs = (int64_t)(bm / 32) * (bn / 32);
    // (only tiles whose waves each own a block have the block kernel: the kernel header's QuadOf)
    if (subs > 1 && bm * bn <= 128 * 64 && bm % 32 == 0 && bn % 32 == 0 && kShapes[tile].waves_k == 1 && !hooks.no_quad) {
        // (whole rounds of blocks: with 272 blocks some compute unit gets two.  The first round fills in behind the
        // whole tiles; every further one costs the blocks' own time, 4 ns per column of K: 512 x 6144 x 4096 in
        // 64 x 128 tiles, 1024 blocks, 72 us)
        const double block_rounds = (double)cdiv(t.tail * subs, 256);
        quad_benefit = t_full - (5.0 * block_rounds + (0.0018 + 0.004 * (block_rounds - 1.0)) * (double)K);
    }
    double range_benefit = 0.0;
    if (S > 1 && t.tail * S * bm * bn * 4 <= kMaxWorkspaceBytes) {
        // measured on launches of 30 us to 3 ms: the second pass adds its launch, 6 us, and the partial products
        // written and read back at 5 TB/s.  The pieces follow the whole tiles, which end within a window of about
        // 20 us where two workgroups share a compute unit (5 us for the tile that has one to itself), and what
        // a piece takes beyond that window is added to the launch (128 x 128 tiles, K = 4096: 16 tail tiles in 8
        // pieces add 7 us of a piece's 30, 65 in 3 add 57 of 77, 128 in 2 add 102 of 114; 2048 x 11008 x 4096:
        // 88 tail tiles of 256 x 256 in two pieces add 450 us to the 920 us of the whole round, a piece taking 459)
        const double t_piece = tile_us(vm, bm, bn, (double)units_per_piece * bk, true);
        const double second_pass = 6.0 + (double)(S + 1) * (double)t.tail * bm * bn * 4.0 / 5.0e6;
        const double added = std::max(0.25 * t_piece, t_piece - (bm * bn >= 256 * 256 ? 5.0 : 20.0));
        range_benefit = t_full - (second_pass + added);
    }
    if (quad_benefit > 0.0 && quad_benefit >= range_benefit) {
        t.pieces = subs;
        t.benefit_us = quad_benefit;
        t.quad = true;
    } else if (range_benefit > 0.0) {
        t.pieces = S;
        t.piece_k = units_per_piece * bk;
        t.benefit_us = range_benefit;
    }
    return t;
}

// set around one call by run_forced: tile and split given by the caller instead of the cost model
thread_local int g_forced_tile = -1, g_forced_split = -1;

Choice evaluate_candidates(const Hooks &hooks, int forced_tile, int forced_split, int64_t batch, int64_t M, int64_t N,
                           int64_t K, int bmode, int amode);

// The cost model walks every (tile, split) candidate: 1-2 us, as much as the launch itself for a small
// product.  A caller repeats a few shapes; each thread remembers the choices of the last ones it asked for.
struct ChoiceKey {
    int64_t batch, M, N, K;
    int bmode, amode, forced_tile, forced_split, flags;
    bool operator==(const ChoiceKey &o) const
    {
        return batch == o.batch && M == o.M && N == o.N && K == o.K && bmode == o.bmode && amode == o.amode &&
               forced_tile == o.forced_tile && forced_split == o.forced_split && flags == o.flags;
    }
};
struct ChoiceSlot { ChoiceKey key; Choice choice; bool valid; };
std::atomic<long long> g_strategy_applied{0}, g_strategy_failed{0};
// Behind the per-thread slots, one table for the process: realising a choice through the strategy layer
// costs about 0.1 ms, which a shape should pay once, not once per thread or per eviction.
struct ChoiceKeyHash {
    size_t operator()(const ChoiceKey &k) const
    {
        uint64_t h = (uint64_t)k.M * 0x9E3779B97F4A7C15ull;
        h = (h ^ (uint64_t)k.N) * 0xC2B2AE3D27D4EB4Full;
        h = (h ^ (uint64_t)k.K) * 0x165667B19E3779F9ull;
        h = (h ^ (uint64_t)k.batch) * 0x27D4EB2F165667C5ull;
        h ^= (uint64_t)(k.bmode | (k.amode << 2) | (k.flags << 4)) ^ ((uint64_t)(uint32_t)k.forced_tile << 16) ^ ((uint64_t)(uint32_t)k.forced_split << 32);
        return (size_t)(h ^ (h >> 29));
    }
};
std::mutex g_choice_mutex;
std::unordered_map<ChoiceKey, Choice, ChoiceKeyHash> g_choice_table;
constexpr size_t kChoiceTableMax = 1u << 16;
thread_local ChoiceSlot g_choice_cache[64];

Choice choose_tile(const Hooks &hooks, int64_t batch, int64_t M, int64_t N, int64_t K, int bmode = B_NN, int amode = A_MK)
{
    const int forced_tile = hooks.force_tile >= 0 ? hooks.force_tile : g_forced_tile;
    const int forced_split = hooks.force_split >= 1 ? hooks.force_split : g_forced_split;
    const ChoiceKey key = {batch, M, N, K, bmode, amode, forced_tile, forced_split,
                           (hooks.no_tail_split ? 1 : 0) | (hooks.no_quad ? 2 : 0) | (hooks.no_kshare ? 4 : 0) | (hooks.no_strip ? 8 : 0) | (hooks.force_strip ? 16 : 0)};
    const uint64_t h = ((uint64_t)M * 0x9E3779B97F4A7C15ull) ^ ((uint64_t)N * 0xC2B2AE3D27D4EB4Full) ^
                       ((uint64_t)K * 0x165667B19E3779F9ull) ^ ((uint64_t)batch * 0x27D4EB2F165667C5ull);
    ChoiceSlot &slot = g_choice_cache[h >> 58];
    if (slot.valid && slot.key == key) return slot.choice;
    {
        std::lock_guard<std::mutex> lock(g_choice_mutex);
        const auto it = g_choice_table.find(key);
        if (it != g_choice_table.end()) {
            slot.key = key;
            slot.choice = it->second;
            slot.valid = true;
            return slot.choice;
        }
    }
    slot.valid = false;
    slot.key = key;
    slot.choice = evaluate_candidates(hooks, forced_tile, forced_split, batch, M, N, K, bmode, amode);
    // The choice is then realised by the strategy layer: a left choice over the tiles, each guarded by "may
    // compete" and "is the cheapest", whose schedule rewrites the product's loop nest; the configuration
    // lowered from the rewritten nest is what the plan is built from.  (Forced tiles and splits are explicit
    // schedules of the caller's; batched products are one nest per batch and keep the model's answer.)
    if (forced_tile < 0 && forced_split < 1 && batch == 1 && M >= 1 && N >= 1 && K >= 1) {
        const TileShape &sh = kShapes[slot.choice.tile];
        const ShapeQuery q = {batch, M, N, K, bmode, amode};
        const TileChoice want = {sh.bm, sh.bn, sh.bk, sh.waves_m, sh.waves_n, sh.waves_k, slot.choice.split};
        TileChoice got;
        int tile = -1;
        if (dispatch_by_strategy(q, want, got))
            for (int t = 0; t < NUM_TILES; ++t)
                if (kShapes[t].bm == got.bm && kShapes[t].bn == got.bn && kShapes[t].bk == got.bk &&
                    kShapes[t].waves_m == got.waves_m && kShapes[t].waves_n == got.waves_n && kShapes[t].waves_k == got.waves_k)
                    tile = t;
        // (the lowered nest counts the K ranges that are not empty; the plan derives the same count from the split)
        const int64_t k_range = cdiv(cdiv(K, slot.choice.split), sh.bk) * sh.bk;
        if (tile >= 0 && got.split == (slot.choice.split > 1 ? (int)cdiv(K, k_range) : 1)) {
            slot.choice = {tile, slot.choice.split, slot.choice.strip};
            g_strategy_applied.fetch_add(1, std::memory_order_relaxed);
        } else {
            g_strategy_failed.fetch_add(1, std::memory_order_relaxed);     // the model's answer stands
        }
    }
    slot.valid = true;
    {
        std::lock_guard<std::mutex> lock(g_choice_mutex);
        if (g_choice_table.size() >= kChoiceTableMax) g_choice_table.clear();
        g_choice_table.emplace(key, slot.choice);
    }
    return slot.choice;
}

// Which tiles may compete for a shape at all (measured rules; the cost model ranks the rest).
bool admissible(const Hooks &hooks, int tile, int64_t batch, int64_t M, int64_t N, int64_t K, int bmode, int amode)
{
    // the 32-wide tiles move a quarter more operand bytes per flop than the 64-wide ones: they
    // are for outputs that are no wider, where the others would compute padding
    // (measured: beyond one round of workgroups they still pay where their tile count fits the chip better,
    // 1100^3 25 against 30 us; they stay out of outputs of more than 2048 tiles, where the traffic counts)
    if (((tile == T128x32 && N > 32) || (tile == T32x128 && M > 32)) &&
        cdiv(M, kShapes[tile].bm) * cdiv(N, kShapes[tile].bn) > 2048) return false;
    // One 32 x 32 block per workgroup with the slab shared between its waves: for outputs at most 32
    // wide whose operands need no element-wise masking (a B stored K x N with fewer than 32 columns
    // does, and so does an A stored K x M with fewer than 32 rows).  Where it
    // applies it replaces the other 32-wide tiles (fewer or no K ranges over workgroups, so no or
    // a smaller second pass): measured 5-20 % faster on such shapes.
    const bool narrow_n = N <= 32 && amode == A_MK && (bmode != B_NN || N == 32) && M >= 1024;
    // (a B stored K x N is read in panels of 32 columns, 128 bytes per row: fine from the memory-side
    // cache, slower than the 128-column tile once B is larger than that cache and streams from HBM:
    // 32 x 32000 x 4096: 125 us against 96)
    const bool b_streams_narrow = bmode == B_NN && M <= 32 && 4.0 * (double)K * (double)N > 268435456.0;
    const bool narrow_m = M <= 32 && (amode == A_MK || M == 32) && N >= 1024 && !b_streams_narrow;
    const bool kshare = batch == 1 && (narrow_n || narrow_m);
    if (tile != TQ32 && kshare) return false;
    // It also competes on any product at least 32 x 32: a few hundred blocks occupy the chip
    // where the same output in 64-wide tiles needs K ranges and a second pass (640 x 640 x 1024:
    // 11.7 instead of 19.4 us).
    // (batched products too: they cannot split K; and batches of products no larger than one block,
    // where a 64 x 64 tile would compute four times the padding: 4096 x 16x16x64 29 -> 20 us)
    const bool kshare_general = ((M >= 32 && N >= 32) || (batch > 1 && M <= 32 && N <= 32)) && !hooks.no_kshare;
    if (tile == TQ32 && ((!kshare && !kshare_general) || b_streams_narrow)) return false;
    // The same with two blocks per workgroup (a quarter fewer operand bytes per flop, half the
    // workgroups): where the output has enough of them (640 x 640 x 2048 with B stored N x K:
    // 21 -> 18.3 us).
    if ((tile == TQ64x32 || tile == TQ32x64) && (kshare || !kshare_general || b_streams_narrow)) return false;
    return true;
}

Choice evaluate_candidates(const Hooks &hooks, int forced_tile, int forced_split, int64_t batch, int64_t M, int64_t N,
                           int64_t K, int bmode, int amode)
{
    Choice best = {TB64, 1, 0};
    double best_cost = -1, best_area = 0;
    for (const auto &c : kCandidates) {
        if (forced_tile >= 0 ? c.id != forced_tile : !admissible(hooks, c.id, batch, M, N, K, bmode, amode)) continue;
        const TileShape &sh = kShapes[c.id];
        const int strip_max = strip_cols(hooks, c.id, batch, N, bmode, amode);   // only without K ranges
        const int64_t tiles_whole = batch * cdiv(M, sh.bm) * cdiv(N, sh.bn);
        static const int kSplits[] = {1, 2, 3, 4, 5, 6, 8, 10, 12, 16, 24, 32, 48, 64, 96, 128, 192, 256, 384, 512};
        // (a shape that allows a strip is tried with it and, its last columns an edge tile column, without)
        for (int si = (strip_max > 0 ? -1 : 0); si < (int)(sizeof(kSplits) / sizeof(kSplits[0])); ++si) {
            int S = si < 0 ? 1 : kSplits[si];
            if (forced_split >= 1) S = forced_split;
            const int strip = (si < 0 && S == 1) ? strip_max : 0;
            if (si < 0 && S != 1) continue;
            if (hooks.force_strip && strip_max > 0 && si >= 0 && S == 1) continue;
            if (S > 1) {
                // every range holds whole slabs and at least two of them; one product only
                if (batch != 1 || K < (int64_t)S * 2 * sh.bk) break;
                if ((int64_t)S * M * N * 4 > kMaxWorkspaceBytes) break;
            }
            const double k_range = (double)cdiv(cdiv(K, S), sh.bk) * sh.bk;
            const int64_t tiles = (S == 1 && strip > 0) ? cdiv(M, sh.bm) * (N / sh.bn) : tiles_whole;
            const int64_t wgs = tiles * S;
            // two workgroups of the two-block shared-slab tiles fit a compute unit; measured, they pay while all
            // of them are resident at once (1024^3: 512 workgroups, 19.3 us) and not beyond (648 x 3072 x 752:
            // 1008 workgroups, 42 us against 31 for 64 x 128 tiles)
            if (forced_tile < 0 && (c.id == TQ64x32 || c.id == TQ32x64) && wgs > 512) continue;
            double cost = (double)cdiv(wgs, 256) * tile_us(c, sh.bm, sh.bn, k_range, wgs > 256);
            // what a launch pays once (start-up, first loads, last stores) is part of the single-round
            // overhead; with several rounds it is still paid once, on top of the per-round overheads
            if (wgs > 256) cost += 2.0 * sh.bm * sh.bn * (c.overhead_single - c.overhead_multi) / (kCuFlopsPerUs * c.single);
            // a matrix shorter than the tile cannot move its edge tiles inside: every tile then runs
            // the masked loads, which cost about a quarter more
            if (M < sh.bm || N < sh.bn) cost *= 1.25;
            // Measured: the 64 x 64 tiles sustain the `multi` rate while only some compute units hold two of them
            // (256 x 5120 x 5120, 320 tiles: 99 us, the best tile); with two on every compute unit they fall 4 %
            // behind it (512 x 4096 x 11008, 512 tiles: 320 us against 308 for 64 x 128 tiles; 4096^3: 979 us).
            if ((c.id == TB64 || c.id == T64) && wgs > 320) cost *= 1.0 + 0.04 * std::min(1.0, (double)(wgs - 320) / 192.0);
            // Measured on ten large shapes: while both operands fit the 256 MB memory-side cache with room to spare,
            // several rounds of 128 x 128 tiles, two workgroups to a compute unit, overlap their epilogues and
            // the drain of C with each other's slab loops and come out 0.4-1.8 % ahead of rounds of the 256-wide
            // tiles (4096^3: 903 against 912 us, 4096 x 4096 x 1024: 233 against 237, 6144^3: 3059 against 3069);
            // at 8192^3 (512 MB of operands) the large tile is 1 % ahead again (7191 against 7266 us).
            if (sh.bm * sh.bn >= 256 * 128 && 4.0 * (double)batch * ((double)M * K + (double)K * N) <= 320.0e6) cost *= 1.012;
            // both operands cross the memory interface at least once, at 5.2 TB/s at best: what
            // bounds products with one short dimension
            // (a workgroup keeps about 40 KB in flight, which at the memory latency is 22 GB/s: fewer
            // than 240 workgroups do not reach the full rate)
            const double bytes_per_us = std::min(5.2e6, (double)wgs * 0.022e6);
            const double hbm_us = 4.0 * (double)batch * ((double)M * K + (double)K * N) / bytes_per_us;
            // (between candidates that are all bound by the memory interface, the one with less matrix work
            // and fewer fixed costs is still the faster: a small share of the compute cost breaks the tie)
            cost = std::max(cost, hbm_us + 0.02 * cost);
            if (S > 1) cost += 7.5 + (double)(S + 1) * M * N * 4.0 / 5.0e6;   // second pass: launch + traffic at 5 TB/s
            // the strip runs beside the tiles, most of it while they wait for their first slab, which it delays
            // (measured against the same product without the last columns: 1.3 us at K = 1000), so it pays where
            // it saves a round of tiles or a split one, not where the edge tile column fits the last round
            // anyway.  A tile that fills a compute unit's registers leaves it no room, and it runs after the tiles.
            if (strip > 0) cost += (sh.bm * sh.bn >= 256 * 256) ? 6.0 + 0.002 * (double)K : 1.5;
            if (S == 1) cost -= plan_tail_split(hooks, c.id, batch, tiles, K).benefit_us;
            // equal cost (the two orientations of a tile on the same number of rounds): the one that
            // computes less padding
            const double area = (double)wgs * sh.bm * sh.bn;
            // (a later candidate has to be more than 1 % cheaper: the model is no more exact than that, and
            // the candidates come largest tile first, fewest K ranges first, which move the fewest bytes)
            if (best_cost < 0 || cost < 0.99 * best_cost || (cost == best_cost && area < best_area)) {
                best_cost = cost;
                best_area = area;
                best = {c.id, S, strip};
            }
            if (forced_split >= 1 && si >= 0) break;
        }
    }
    if (best_cost < 0 && forced_tile >= 0) best = {forced_tile, 1, 0};   // forced split did not fit: no split
    if (batch == 1 && M <= 64 && N <= 64 && K <= 64 && forced_tile < 0) best = {TB64, 1, 0};
    return best;
}

int choose_group_m(int tiles_m, int tiles_n, int64_t total)
{
    // each XCD walks total/8 consecutive tiles; aim for a square run
    int64_t per_xcd = total / 8;
    if (per_xcd < 1) per_xcd = 1;
    int g = 1;
    while ((int64_t)(2 * g) * (2 * g) <= per_xcd && 2 * g <= tiles_m) g *= 2;
    (void)tiles_n;
    return g;
}

struct Plan {
    int status;
    bool launch;
    int bmode, amode, tile;
    float alpha, beta;   // the caller's; args carries (1, 0) when a second pass applies them
    int split;           // K ranges (1: no split)
    int tail_tiles;      // tiles of the last round that are split along K (0: none)
    int64_t user_ldc;    // leading dimension of the caller's C (args.ldc is the workspace's when split)
    bool vec;
    int thin;            // 0: tiles; 1: at most 8 rows, B streamed by the vector-unit kernel; 2: at most 8 columns, A streamed
    size_t workspace_bytes;   // what the launch needs besides the operands (0: nothing)
    int strip;                // columns of C computed by the strip workgroups (0: none)
    KArgs args;
};

// Workspace: the partial products of a K split (S dense M x N matrices) or of a split last round
// (dense BM x BN tiles).  One buffer per (device, stream), so calls on different streams never share
// one; calls on one stream are ordered by the stream.  A buffer that is too small is replaced by a
// larger one (at least twice its size); the old one may still be read by work already enqueued, so it
// is kept until gemm_f32_shutdown: no call ever frees memory or waits for the device.
struct Workspace { int device; hipStream_t stream; float *ptr; size_t bytes; };
std::mutex g_workspace_mutex;
std::vector<Workspace> g_workspaces;
std::vector<void *> g_retired;

int acquire_workspace(size_t bytes, float **out)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail_hip(e);
    std::lock_guard<std::mutex> lock(g_workspace_mutex);
    Workspace *w = nullptr;
    for (auto &cand : g_workspaces)
        if (cand.device == dev && cand.stream == g_stream) w = &cand;
    if (w == nullptr) {
        g_workspaces.push_back(Workspace{dev, g_stream, nullptr, 0});
        w = &g_workspaces.back();
    }
    if (bytes > w->bytes) {
        size_t want = std::max(bytes, std::min<size_t>(2 * w->bytes, (size_t)kMaxWorkspaceBytes));
        want = (want + 65535) & ~(size_t)65535;
        float *fresh = nullptr;
        e = hipMalloc(reinterpret_cast<void **>(&fresh), want);
        if (e != hipSuccess) {
            (void)hipGetLastError();
            g_last_hip_error = (int)e;
            return GEMMF32_ENOMEM;
        }
        if (w->ptr != nullptr) g_retired.push_back(w->ptr);
        w->ptr = fresh;
        w->bytes = want;
    }
    *out = w->ptr;
    return GEMMF32_OK;
}

// Scratch of the entry point that allocates nothing: a fixed array in the code object, one copy per
// device.  Host code must not use the array's name as an address; the device address is looked up once
// per device, with that device current.
constexpr int kMaxDevices = 64;
std::atomic<float *> g_scratch_ptr[kMaxDevices];

int static_scratch(float **out)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail_hip(e);
    if (dev < 0 || dev >= kMaxDevices) return GEMMF32_EINVAL;
    float *ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (ptr == nullptr) {
        e = hipGetSymbolAddress(reinterpret_cast<void **>(&ptr), HIP_SYMBOL(scratch));
        if (e != hipSuccess || ptr == nullptr) return fail_hip(e != hipSuccess ? e : hipErrorInvalidSymbol);
        g_scratch_ptr[dev].store(ptr, std::memory_order_release);
    }
    *out = ptr;
    return GEMMF32_OK;
}

int check_common(int64_t batch, int64_t M, int64_t N, int64_t K, const float *A, int64_t lda, int amode,
                 const float *B, const float *C, int64_t ldc)
{
    if (batch < 0 || M < 0 || N < 0 || K < 0) return GEMMF32_EINVAL;
    if (M > kMaxDim || N > kMaxDim || K > kMaxDim || batch > kMaxDim) return GEMMF32_EINVAL;
    const int64_t a_rows = (amode == A_KM) ? K : M, a_cols = (amode == A_KM) ? M : K;
    if (lda < (a_cols > 1 ? a_cols : 1) || ldc < (N > 1 ? N : 1)) return GEMMF32_EINVAL;
    if (a_rows * lda > kMaxElems || M * ldc > kMaxElems) return GEMMF32_EINVAL;
    const bool has_out = batch > 0 && M > 0 && N > 0;
    if (has_out && C == nullptr) return GEMMF32_ENULL;
    if (has_out && K > 0 && (A == nullptr || B == nullptr)) return GEMMF32_ENULL;
    if (has_out && (C == A || C == B)) return GEMMF32_EALIAS;
    return GEMMF32_OK;
}

Plan make_plan(int64_t batch, int64_t M, int64_t N, int64_t K, const float *A, int64_t lda, int64_t sA,
               const float *B, int64_t ldb, int64_t sB, float *C, int64_t ldc, int64_t sC, int bmode,
               int amode = A_MK, float alpha = 1.f, float beta = 0.f)
{
    Plan pl;
    std::memset(&pl, 0, sizeof(pl));
    pl.bmode = bmode;
    pl.amode = amode;
    pl.alpha = alpha;
    pl.beta = beta;
    pl.status = check_common(batch, M, N, K, A, lda, amode, B, C, ldc);
    if (pl.status != GEMMF32_OK) return pl;
    if (amode == A_KM && bmode == B_PACKED) { pl.status = GEMMF32_EINVAL; return pl; }
    if (bmode == B_NN && ldb < (N > 1 ? N : 1)) { pl.status = GEMMF32_EINVAL; return pl; }
    if (bmode == B_NT && ldb < (K > 1 ? K : 1)) { pl.status = GEMMF32_EINVAL; return pl; }
    if (bmode != B_PACKED && (bmode == B_NN ? K : N) * ldb > kMaxElems) { pl.status = GEMMF32_EINVAL; return pl; }
    if (batch > 1 && (sA < 0 || sB < 0 || sC < 0)) { pl.status = GEMMF32_EINVAL; return pl; }
    if (batch == 0 || M == 0 || N == 0) return pl;  // nothing to do


    const Hooks hooks = read_hooks();
    const Choice ch = choose_tile(hooks, batch, M, N, K, bmode, amode);
    pl.tile = ch.tile;
    pl.split = ch.split;
    // At most 4 rows or columns, both operands with k contiguous, a long side too short to give 256 blocks of
    // 32 and a long operand of at least 160 MB: streamed by the vector-unit kernel instead of 32-wide tiles
    // with K ranges and a second pass.  Measured on both sides of each bound: 4 x 4096 x 11008 (180 MB) 28.5 us
    // this way against 32.9 with tiles, 4 x 4096 x 8192 (134 MB) 29.6 against 23.5; 8192 or more rows in the
    // long operand (256 blocks without K ranges) 48-53 against 39-42; 6 and 8 rows 48-74 against 23-42 (the
    // short operand's loads through the caches then outweigh the stream).
    pl.thin = 0;
    if (batch == 1 && bmode == B_NT && amode == A_MK && K >= 1 && !hooks.no_thin && hooks.force_tile < 0 &&
        hooks.force_split < 0 && g_forced_tile < 0 && g_forced_split < 0) {
        const bool force_thin = hooks.force_thin;       // test hook: whenever it can run
        if (M <= 8 && N >= 64 && (force_thin || (M <= 4 && N < 8192 && N * K >= (40LL << 20)))) pl.thin = 1;
        else if (N <= 8 && M >= 64 && (force_thin || (N <= 4 && M < 8192 && M * K >= (40LL << 20)))) pl.thin = 2;
    }
    if (pl.thin != 0) pl.split = 1;             // the arguments below stay those of the whole product
    const int bm = kShapes[pl.tile].bm, bn = kShapes[pl.tile].bn;
    // (the strip addresses a row of A and a chunk of 1024 rows of B through 32-bit offsets)
    const bool strip_fits = K < (1LL << 30) && (bmode != B_NN || ldb < (1LL << 20));
    const int strip = (pl.split == 1 && pl.thin == 0 && strip_fits) ? ch.strip : 0;
    const int64_t tiles_m = cdiv(M, bm), tiles_n = strip > 0 ? N / bn : cdiv(N, bn);
    const int64_t total = (pl.split > 1 ? pl.split : batch) * tiles_m * tiles_n;
    if (total > kMaxDim) { pl.status = GEMMF32_EINVAL; return pl; }

    bool vec = aligned16(A) && aligned16(C) && lda % 4 == 0 && ldc % 4 == 0;
    if (bmode != B_PACKED) vec = vec && aligned16(B) && ldb % 4 == 0;
    if (batch > 1) vec = vec && sA % 4 == 0 && sC % 4 == 0 && (bmode == B_PACKED || sB % 4 == 0);
    pl.vec = vec;

    pl.user_ldc = ldc;
    KArgs &a = pl.args;
    a.A = A; a.B = B; a.C = C;
    a.M = (int)M; a.N = (int)(N - strip); a.K = (int)K;        // with a strip the tiles end where it begins
    a.lda = lda; a.ldb = ldb; a.ldc = ldc;
    a.sA = sA; a.sB = sB; a.sC = sC;
    set_tile_walk(a, (int)tiles_m, (int)tiles_n, choose_group_m((int)tiles_m, (int)tiles_n, batch > 1 ? tiles_m * tiles_n : total));
    a.total_tiles = (int)total;
    a.n_padded = (int)(cdiv(N, kPanel) * kPanel);
    a.k_total = 0;
    a.k_panel = (int)K;
    a.tail_first = (int)total;
    a.tail_split = 1;
    a.tail_k = 0;
    a.tail_slots = nullptr;
    a.quad = 0;
    a.alpha = alpha;
    a.beta = beta;
#ifdef GEMMF32_TIMELINE
    a.stamps = g_timeline_stamps;
#endif
    pl.tail_tiles = 0;
    // Split tail: when the last round of tiles would leave most compute units idle, its tiles are
    // cut along K so that the round fills the chip (272 tiles = one full round + 16 tiles -> those
    // 16 become 256 pieces that run beside the full round).
    if (pl.split == 1 && pl.thin == 0) {
        const TailSplit ts = plan_tail_split(hooks, pl.tile, batch, total, K);
        if (ts.pieces > 1) {
            a.tail_first = (int)(total - ts.tail);
            a.tail_split = (int)ts.pieces;
            a.tail_k = (int)ts.piece_k;
            a.total_tiles = (int)(total - ts.tail + ts.tail * ts.pieces);
            a.quad = ts.quad ? 1 : 0;
            pl.tail_tiles = (int)ts.tail;
        }
    }
    if (pl.split > 1) {
        // K ranges of whole slabs; range s starts k_range columns (rows of B) after range s-1 and
        // writes the dense partial product s of the workspace (pointer filled in by run_plan)
        const int bk = kShapes[pl.tile].bk;
        const int64_t k_range = cdiv(cdiv(K, pl.split), bk) * bk;
        pl.split = (int)cdiv(K, k_range);           // ranges that are not empty
        a.K = (int)k_range;
        a.k_total = (int)K;
        a.sA = (amode == A_KM) ? k_range * lda : k_range;
        a.sB = (bmode == B_NN) ? k_range * ldb : (bmode == B_NT ? k_range : k_range * kPanel);
        a.sC = M * N;
        a.ldc = N;
        a.total_tiles = (int)(pl.split * tiles_m * tiles_n);
        a.alpha = 1.f;                  // raw partial sums; the second pass applies alpha and beta
        a.beta = 0.f;
        if (pl.split == 1) {
            a.K = (int)K; a.k_total = 0; a.sA = a.sB = a.sC = 0; a.ldc = ldc; a.alpha = alpha; a.beta = beta;
        }
    }
    a.strip_first = a.total_tiles;
    pl.strip = strip;
    if (strip > 0) {
        a.strip_cols = strip;
        a.strip_n0 = (int)(N - strip);
        // 1, 2 or 4 rows per wave (measured: one row up to 512 rows of C, two up to 2048: 1024 x 1028 x 1024 19.1 us
        // against 19.6 with one, 1536 x 1541 x 1536 56.5 against 60.8; four beyond: 4096 x 4100 x 4096 910 against 916)
        a.strip_r = M <= 512 ? 1 : (M <= 2048 ? 2 : 4);
        if (hooks.strip_rows > 0) a.strip_r = hooks.strip_rows;
        a.strip_wait = hooks.strip_wait >= 0 ? hooks.strip_wait : 0;
        const int64_t strip_wgs = cdiv(M, 4 * a.strip_r);
        if ((int64_t)a.total_tiles + strip_wgs > kMaxDim) { pl.status = GEMMF32_EINVAL; return pl; }
        a.total_tiles += (int)strip_wgs;
    }
    if (pl.split > 1) pl.workspace_bytes = (size_t)pl.split * (size_t)M * (size_t)N * sizeof(float);
    else if (pl.tail_tiles > 0 && a.quad == 0)
        pl.workspace_bytes = (size_t)pl.tail_tiles * a.tail_split * kShapes[pl.tile].bm * kShapes[pl.tile].bn * sizeof(float);
    pl.launch = true;
    return pl;
}

// second pass of a K split: sums `split` dense M x N partial products from W into C
int launch_splitk_reduce(const float *W, float *C, int M, int N, int64_t ldc, int split, float alpha, float beta)
{
    // lanes per group of 4 columns: enough to put about 64K threads on the chip, at most 64, at most S
    const int64_t chunks = (int64_t)M * ((N + 3) / 4);
    int sl = 1;
    while (sl < 64 && sl * 2 <= split && chunks * sl < 65536) sl *= 2;
    const dim3 grid((unsigned)cdiv(chunks * sl, 256)), block(256);
    switch (sl) {
    case 1: hipLaunchKernelGGL(splitk_reduce_kernel<1>, grid, block, 0, g_stream, W, C, M, N, ldc, split, alpha, beta); break;
    case 2: hipLaunchKernelGGL(splitk_reduce_kernel<2>, grid, block, 0, g_stream, W, C, M, N, ldc, split, alpha, beta); break;
    case 4: hipLaunchKernelGGL(splitk_reduce_kernel<4>, grid, block, 0, g_stream, W, C, M, N, ldc, split, alpha, beta); break;
    case 8: hipLaunchKernelGGL(splitk_reduce_kernel<8>, grid, block, 0, g_stream, W, C, M, N, ldc, split, alpha, beta); break;
    case 16: hipLaunchKernelGGL(splitk_reduce_kernel<16>, grid, block, 0, g_stream, W, C, M, N, ldc, split, alpha, beta); break;
    case 32: hipLaunchKernelGGL(splitk_reduce_kernel<32>, grid, block, 0, g_stream, W, C, M, N, ldc, split, alpha, beta); break;
    default: hipLaunchKernelGGL(splitk_reduce_kernel<64>, grid, block, 0, g_stream, W, C, M, N, ldc, split, alpha, beta); break;
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail_hip(e);
    return GEMMF32_OK;
}

template <int S> int launch_thin_s(const ThinArgs &t)
{
    hipLaunchKernelGGL(thin_nt_kernel<S>, dim3((unsigned)cdiv(t.rows, kThinRowsPerWorkgroup)), dim3(256), 0, g_stream, t);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail_hip(e);
    return GEMMF32_OK;
}

int launch_thin(const Plan &pl)
{
    const KArgs &a = pl.args;
    ThinArgs t;
    t.K = a.K;
    t.alpha = pl.alpha;
    t.beta = pl.beta;
    t.C = a.C;
    int small;
    if (pl.thin == 1) {          // C[m][n]: n runs over the streamed rows of B
        t.X = a.B; t.ldx = a.ldb; t.rows = a.N; t.Y = a.A; t.ldy = a.lda; t.c_big = 1; t.c_small = pl.user_ldc; small = a.M;
    } else {                     // m runs over the streamed rows of A
        t.X = a.A; t.ldx = a.lda; t.rows = a.M; t.Y = a.B; t.ldy = a.ldb; t.c_big = pl.user_ldc; t.c_small = 1; small = a.N;
    }
    switch (small) {
    case 1: return launch_thin_s<1>(t);
    case 2: return launch_thin_s<2>(t);
    case 3: return launch_thin_s<3>(t);
    case 4: return launch_thin_s<4>(t);
    case 5: return launch_thin_s<5>(t);
    case 6: return launch_thin_s<6>(t);
    case 7: return launch_thin_s<7>(t);
    case 8: return launch_thin_s<8>(t);
    default: return GEMMF32_EINVAL;
    }
}

// static_only: the workspace is the fixed scratch array and nothing is allocated
int run_plan(const Plan &pl, bool static_only = false)
{
    if (pl.status != GEMMF32_OK) return pl.status;
    if (!pl.launch) return GEMMF32_OK;
    if (pl.thin != 0) return launch_thin(pl);
    float *workspace = nullptr;
    if (pl.workspace_bytes > 0) {
        if (static_only && pl.workspace_bytes > kScratchBytes) return GEMMF32_ESCRATCH;
        const int rc = static_only ? static_scratch(&workspace) : acquire_workspace(pl.workspace_bytes, &workspace);
        if (rc != GEMMF32_OK) return rc;
    }
    if (pl.split <= 1 && pl.tail_tiles > 0 && pl.args.quad == 0) {
        const TileShape &sh = kShapes[pl.tile];
        KArgs a = pl.args;
        a.tail_slots = workspace;
        const int rc = launch_variant(pl.bmode, pl.amode, pl.tile, a);
        if (rc != GEMMF32_OK) return rc;
        hipLaunchKernelGGL(tail_reduce_kernel, dim3((unsigned)(pl.tail_tiles * (sh.bm * sh.bn / 256))), dim3(64), 0,
                           g_stream, a, sh.bm, sh.bn);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return fail_hip(e);
        return GEMMF32_OK;
    }
    if (pl.split <= 1) return launch_variant(pl.bmode, pl.amode, pl.tile, pl.args);
    // split K: partial products into the workspace, then one pass that sums them in order
    KArgs a = pl.args;
    float *C = a.C;
    const int64_t ldc = pl.user_ldc;
    a.C = workspace;
    const int rc = launch_variant(pl.bmode, pl.amode, pl.tile, a);
    if (rc != GEMMF32_OK) return rc;
    return launch_splitk_reduce(workspace, C, a.M, a.N, ldc, pl.split, pl.alpha, pl.beta);
}

thread_local char g_variant_buf[64];

// Nothing but matrix instructions: every wave issues `steps` rounds of 16 MFMAs on four independent
// accumulators from registers.  One MFMA 32x32x2 occupies a SIMD's matrix pipe for 64 cycles, so the
// run time gives the clock the chip sustains under full matrix load.  The operands come from
// operands[2*lane], operands[2*lane + 1]: the sustained clock depends on their values (zeros draw
// less power than random numbers).
__global__ void __launch_bounds__(256, 1) mfma_rate_kernel(int steps, const float *operands, float *sink)
{
    v16f acc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
    const float a = operands[2 * threadIdx.x], b = operands[2 * threadIdx.x + 1];
    for (int s = 0; s < steps; ++s) {
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int i = 0; i < 4; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc[i], 0, 0, 0);
    }
    float t = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) t += acc[i][v];
    if (t == -1.f) sink[0] = t;          // never true; keeps the accumulators alive
}

}  // namespace

namespace gemmf32_host {

TileChoice choose(int64_t M, int64_t N, int64_t K)
{
    const Choice c = choose_tile(read_hooks(), 1, M, N, K);
    const TileShape &sh = kShapes[c.tile];
    int split = c.split;
    if (split > 1) {   // the ranges that are not empty, as make_plan counts them
        const int64_t k_range = cdiv(cdiv(K, split), sh.bk) * sh.bk;
        split = (int)cdiv(K, k_range);
    }
    return TileChoice{sh.bm, sh.bn, sh.bk, sh.waves_m, sh.waves_n, sh.waves_k, split};
}

int tile_count() { return NUM_TILES; }

TileChoice tile_shape(int tile)
{
    const TileShape &sh = kShapes[tile];
    return TileChoice{sh.bm, sh.bn, sh.bk, sh.waves_m, sh.waves_n, sh.waves_k, 1};
}

bool admissible_tile(int tile, const ShapeQuery &q)
{
    return admissible(read_hooks(), tile, q.batch, q.M, q.N, q.K, q.bmode, q.amode);
}

void strategy_dispatch_stats(long long *applied, long long *failed)
{
    if (applied) *applied = g_strategy_applied.load();
    if (failed) *failed = g_strategy_failed.load();
}

bool has_kernel(int bm, int bn, int bk, int waves_m, int waves_n, int waves_k)
{
    for (const TileShape &sh : kShapes)
        if (sh.bm == bm && sh.bn == bn && sh.bk == bk && sh.waves_m == waves_m && sh.waves_n == waves_n &&
            sh.waves_k == waves_k)
            return true;
    return false;
}

int run_forced(int bm, int bn, int bk, int split, int64_t M, int64_t N, int64_t K, const float *A, int64_t lda,
               const float *B, int64_t ldb, float *C, int64_t ldc, int transB)
{
    int tile = -1;
    for (int t = 0; t < NUM_TILES; ++t)
        if (kShapes[t].bm == bm && kShapes[t].bn == bn && kShapes[t].bk == bk) tile = t;
    if (tile < 0 || split < 1 || split > 256) return GEMMF32_EINVAL;
    // a split must leave every range at least two slabs and fit the workspace (what choose_tile requires)
    if (split > 1 && (K < (int64_t)split * 2 * bk || (int64_t)split * M * N * 4 > kMaxWorkspaceBytes)) return GEMMF32_EINVAL;
    if (transB != 0 && transB != 1) return GEMMF32_EINVAL;
    g_forced_tile = tile;
    g_forced_split = split;
    const Plan pl = make_plan(1, M, N, K, A, lda, 0, B, ldb, 0, C, ldc, 0, transB ? B_NT : B_NN);
    g_forced_tile = g_forced_split = -1;
    return run_plan(pl);
}

}  // namespace gemmf32_host

extern "C" {

int gemm_f32(int64_t M, int64_t N, int64_t K, const float *A, int64_t lda, const float *B, int64_t ldb,
             float *C, int64_t ldc, int transB)
{
    if (transB != 0 && transB != 1) return GEMMF32_EINVAL;
    return run_plan(make_plan(1, M, N, K, A, lda, 0, B, ldb, 0, C, ldc, 0, transB ? B_NT : B_NN));
}

int gemm_f32_batched(int64_t batch, int64_t M, int64_t N, int64_t K, const float *A, int64_t lda,
                     int64_t strideA, const float *B, int64_t ldb, int64_t strideB, float *C, int64_t ldc,
                     int64_t strideC, int transB)
{
    if (transB != 0 && transB != 1) return GEMMF32_EINVAL;
    if (M == 64 && N == 64 && K == 64 && batch >= 2 && read_hooks().force_tile < 0) {
        // streaming path for many 64^3 products; same argument checks as the general path
        Plan pl = make_plan(batch, M, N, K, A, lda, strideA, B, ldb, strideB, C, ldc, strideC,
                            transB ? B_NT : B_NN);
        if (pl.status != GEMMF32_OK) return pl.status;
        return launch_batched64(batch, A, lda, strideA, B, ldb, strideB, C, ldc, strideC, transB);
    }
    return run_plan(make_plan(batch, M, N, K, A, lda, strideA, B, ldb, strideB, C, ldc, strideC,
                              transB ? B_NT : B_NN));
}

int gemm_f32_ex(int64_t M, int64_t N, int64_t K, float alpha, const float *A, int64_t lda, int transA,
                const float *B, int64_t ldb, int transB, float beta, float *C, int64_t ldc)
{
    if ((transA != 0 && transA != 1) || (transB != 0 && transB != 1)) return GEMMF32_EINVAL;
    return run_plan(make_plan(1, M, N, K, A, lda, 0, B, ldb, 0, C, ldc, 0, transB ? B_NT : B_NN,
                              transA ? A_KM : A_MK, alpha, beta));
}

int gemm_f32_ex_batched(int64_t batch, int64_t M, int64_t N, int64_t K, float alpha, const float *A, int64_t lda,
                        int64_t strideA, int transA, const float *B, int64_t ldb, int64_t strideB, int transB,
                        float beta, float *C, int64_t ldc, int64_t strideC)
{
    if ((transA != 0 && transA != 1) || (transB != 0 && transB != 1)) return GEMMF32_EINVAL;
    if (!transA && alpha == 1.f && beta == 0.f)
        return gemm_f32_batched(batch, M, N, K, A, lda, strideA, B, ldb, strideB, C, ldc, strideC, transB);
    return run_plan(make_plan(batch, M, N, K, A, lda, strideA, B, ldb, strideB, C, ldc, strideC,
                              transB ? B_NT : B_NN, transA ? A_KM : A_MK, alpha, beta));
}

#ifdef GEMMF32_TIMELINE
// measurement build only: DEVICE buffer of 8 * 4096 64-bit slots that later launches stamp (NULL: off)
int gemm_f32_timeline_set(void *stamps)
{
    g_timeline_stamps = reinterpret_cast<unsigned long long *>(stamps);
    return GEMMF32_OK;
}
#endif

int64_t pack_b_panel_width(void) { return kPanel; }

size_t pack_b_size(int64_t N, int64_t K)
{
    if (N <= 0 || K <= 0) return 0;
    return (size_t)(cdiv(N, kPanel) * K * kPanel) * sizeof(float);
}

int pack_b(int64_t N, int64_t K, const float *B, int64_t ldb, int transB, float *Bp)
{
    if (transB != 0 && transB != 1) return GEMMF32_EINVAL;
    if (N < 0 || K < 0 || N > kMaxDim || K > kMaxDim) return GEMMF32_EINVAL;
    if (transB ? ldb < (K > 1 ? K : 1) : ldb < (N > 1 ? N : 1)) return GEMMF32_EINVAL;
    if ((transB ? N : K) * ldb > kMaxElems) return GEMMF32_EINVAL;
    if (N == 0 || K == 0) return GEMMF32_OK;
    if (B == nullptr || Bp == nullptr) return GEMMF32_ENULL;
    if (B == Bp) return GEMMF32_EALIAS;
    if (!aligned16(Bp)) return GEMMF32_EINVAL;
    if (transB) {
        const int64_t k_blocks = cdiv(K, 64);
        const int64_t blocks = cdiv(N, kPanel) * 2 * k_blocks;
        if (blocks > kMaxDim) return GEMMF32_EINVAL;
        hipLaunchKernelGGL(pack_b_transposed_kernel, dim3((unsigned)blocks), dim3(256), 0, g_stream, B, Bp, (int)N,
                           (int)K, ldb, (int)k_blocks);
    } else {
        const int64_t total_f4 = cdiv(N, kPanel) * K * (kPanel / 4);
        const int64_t blocks = cdiv(total_f4, 1024);
        if (blocks > kMaxDim) return GEMMF32_EINVAL;
        hipLaunchKernelGGL(pack_b_kernel, dim3((unsigned)blocks), dim3(256), 0, g_stream, B, Bp, (int)N, (int)K, ldb,
                           total_f4);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail_hip(e);
    return GEMMF32_OK;
}

int gemm_f32_packed(int64_t M, int64_t N, int64_t K, const float *A, int64_t lda, const float *Bp, float *C,
                    int64_t ldc)
{
    if (Bp != nullptr && !aligned16(Bp)) return GEMMF32_EINVAL;
    return run_plan(make_plan(1, M, N, K, A, lda, 0, Bp, kPanel, 0, C, ldc, 0, B_PACKED));
}

int gemm_f32_mfma_rate_probe(int64_t mfma_per_wave, const float *operands, float *sink)
{
    if (mfma_per_wave < 16 || mfma_per_wave > (1LL << 30) || mfma_per_wave % 16 != 0) return GEMMF32_EINVAL;
    if (sink == nullptr || operands == nullptr) return GEMMF32_ENULL;
    hipLaunchKernelGGL(mfma_rate_kernel, dim3(256), dim3(256), 0, g_stream, (int)(mfma_per_wave / 16), operands, sink);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail_hip(e);
    return GEMMF32_OK;
}

int gemm_f32_set_stream(void *hip_stream)
{
    g_stream = reinterpret_cast<hipStream_t>(hip_stream);
    return GEMMF32_OK;
}

const char *gemm_f32_strerror(int status)
{
    switch (status) {
    case GEMMF32_OK: return "ok";
    case GEMMF32_EINVAL: return "invalid dimension, stride, alignment or flag";
    case GEMMF32_ENULL: return "null pointer";
    case GEMMF32_EALIAS: return "output aliases an input";
    case GEMMF32_ELAUNCH: return "HIP runtime error (see gemm_f32_last_hip_error)";
    case GEMMF32_ENOMEM: return "out of memory";
    case GEMMF32_ESCRATCH: return "the product needs more scratch memory than the allocation-free entry point holds";
    default: return "unknown status";
    }
}

int gemm_f32_last_hip_error(void) { return g_last_hip_error; }

void gemm_f32_shutdown(void)
{
    (void)hipDeviceSynchronize();      // work that still reads a workspace
    std::lock_guard<std::mutex> lock(g_workspace_mutex);
    for (auto &w : g_workspaces)
        if (w.ptr != nullptr) (void)hipFree(w.ptr);
    for (void *p : g_retired) (void)hipFree(p);
    g_workspaces.clear();
    g_retired.clear();
}

int gemm_f32_reserve_workspace(size_t bytes)
{
    if (bytes > (size_t)kMaxWorkspaceBytes) return GEMMF32_EINVAL;
    if (bytes == 0) return GEMMF32_OK;
    float *unused = nullptr;
    return acquire_workspace(bytes, &unused);
}

size_t gemm_f32_noalloc_scratch_bytes(void) { return kScratchBytes; }

int gemm_f32_noalloc(int64_t M, int64_t N, int64_t K, const float *A, int64_t lda, const float *B, int64_t ldb,
                     float *C, int64_t ldc, int transB)
{
    if (transB != 0 && transB != 1) return GEMMF32_EINVAL;
    return run_plan(make_plan(1, M, N, K, A, lda, 0, B, ldb, 0, C, ldc, 0, transB ? B_NT : B_NN), true);
}

int gemm_f32_set_test_hooks(const gemmf32_test_hooks *h)
{
    const gemmf32_test_hooks off = {-1, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
    if (h == nullptr) h = &off;
    if (h->force_tile < -1 || h->force_tile >= NUM_TILES || h->force_split < 0 || h->force_split > 256 ||
        h->strip_wait < 0 || h->strip_wait > 65 || (h->strip_rows != 0 && h->strip_rows != 1 && h->strip_rows != 2 && h->strip_rows != 4))
        return GEMMF32_EINVAL;
    g_hooks.force_tile.store(h->force_tile);
    g_hooks.force_split.store(h->force_split >= 1 ? h->force_split : -1);
    g_hooks.no_tail_split.store(h->no_tail_split != 0);
    g_hooks.no_quad.store(h->no_quad != 0);
    g_hooks.no_kshare.store(h->no_kshare != 0);
    g_hooks.no_thin.store(h->no_thin != 0);
    g_hooks.force_thin.store(h->force_thin != 0);
    g_hooks.no_strip.store(h->no_strip != 0);
    g_hooks.strip_wait.store(h->strip_wait);
    g_hooks.force_strip.store(h->force_strip != 0);
    g_hooks.strip_rows.store(h->strip_rows);
    return GEMMF32_OK;
}

const char *gemm_f32_variant_name(int64_t M, int64_t N, int64_t K, const float *A, int64_t lda, const float *B,
                                  int64_t ldb, const float *C, int64_t ldc, int transB)
{
    // alignment is judged on the pointers' low bits only; nothing is dereferenced
    const float *a = A ? A : reinterpret_cast<const float *>(uintptr_t(16));
    const float *b = B ? B : reinterpret_cast<const float *>(uintptr_t(32));
    float *c = C ? const_cast<float *>(C) : reinterpret_cast<float *>(uintptr_t(48));
    Plan pl = make_plan(1, M, N, K, a, lda, 0, b, ldb, 0, c, ldc, 0, transB ? B_NT : B_NN);
    if (pl.status != GEMMF32_OK) return "invalid";
    if (!pl.launch) return "empty";
    if (pl.thin != 0) {
        std::snprintf(g_variant_buf, sizeof(g_variant_buf), "thin%dx%d/nt", (int)(pl.thin == 1 ? M : N), kThinRows);
        return g_variant_buf;
    }
    int n = std::snprintf(g_variant_buf, sizeof(g_variant_buf), "%s/%s/%s", kShapes[pl.tile].name,
                          pl.bmode == B_NT ? "nt" : "nn", pl.vec ? "a16" : "a4");
    const auto append = [&](const char *fmt, int x, int y) {
        if (n > 0 && n < (int)sizeof(g_variant_buf)) n += std::snprintf(g_variant_buf + n, sizeof(g_variant_buf) - n, fmt, x, y);
    };
    if (pl.tail_tiles > 0 && pl.args.quad != 0) append("/quad%d", pl.tail_tiles, 0);
    else if (pl.tail_tiles > 0) append("/tail%dx%d", pl.tail_tiles, pl.args.tail_split);
    else if (pl.split > 1) append("/splitk%d", pl.split, 0);
    if (pl.strip > 0) append("/strip%d", pl.strip, 0);
    return g_variant_buf;
}

}  // extern "C"
