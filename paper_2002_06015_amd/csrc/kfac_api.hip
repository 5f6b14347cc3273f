// Host side of the C ABI declared in include/kfac.h: argument validation, per-call
// planning (which grouped launches, with which device tables and workspace slices),
// table upload and launch.  Every step of the path runs in the HIP kernels of this
// library; this file only decides what to launch.
#include "../../include/kfac.h"
#include "kfac_internal.h"

#include <algorithm>
#include <climits>
#include <cmath>
#include <cstdint>
#include <cstdlib>
#include <cstring>
#include <functional>
#include <vector>

using namespace kfac;

// ------------------------------------------------------------------ context
namespace {

constexpr int kSlots = 8;
constexpr int kSyncEvents = 12;  // events that order the streams of one call among each other
constexpr size_t kAlign = 256;

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

struct Tunables {
    int target_wgs;      // split-K gives a problem at least this many workgroups (if K allows)
    int min_k_per_split; // never split below this contraction length
    int max_k_per_wg;    // and never leaves a workgroup a longer contraction than this
    int inv_streams;     // independent inversion chains run on this many streams (1..4)
    int rec_leaf;        // the blocked inversion recurses down to blocks of at most this size
    int early_n;         // fused step: layers with a factor of at least this size are built first so
                         // that their inversion chains start while the other factors are still being built
    int corr;            // 1: A factors of 3x3 / stride 1 / pad 1 convolutions through spatial correlations
    int slots;           // staging slots in use (2..kSlots): a call waits until the device has started the
                         // call `slots` calls back.  Measured: letting the host run further ahead than a
                         // couple of calls makes the chains of small launches slower, not faster.
    int pipe;            // fused step: 1 spreads each factor phase over streams (rewrites of the next phase and
                         // reductions of the previous one under the matrix launches of the current one)
    double chunk_gf;     // fused step: matrix launches of the later factor phases in parts of about this many
                         // GFLOP (0: whole)
    int split;           // 1 (default): fp32 products through three bf16 planes and six bf16 matrix instructions
                         // (fp32 accuracy at the bf16 unit's rate); 0: the fp32 matrix instruction
    int force_tile;      // 0: the planner chooses; 64 / 128: every product with that tile
    bool worst_case_splits = false;   // set for the workspace bound: every product split as if it were alone in its launch
    int by_depth;        // kfac_invert: layers grouped onto streams by the length of their chains (1) or by total n^3 (0)
    explicit Tunables(const kfac_options &o)
    {
        target_wgs = std::max(1, o.target_workgroups);
        min_k_per_split = std::max(32, o.min_k_per_split / 32 * 32);
        max_k_per_wg = std::max(32, o.max_k_per_workgroup / 32 * 32);
        inv_streams = std::min(4, std::max(1, o.streams));
        rec_leaf = std::min(kLeafMax, std::max(32, o.recursion_leaf));
        early_n = std::max(1, o.early_n);
        corr = o.correlation_form != 0;
        slots = std::min(kSlots, std::max(2, o.staging_slots));
        pipe = o.pipeline_phases != 0;
        chunk_gf = std::max(0.0f, o.chunk_gflop);
        split = o.fp32_products == KFAC_PRODUCTS_FP32_MFMA ? 0 : 1;
        force_tile = (o.force_tile == 64 || o.force_tile == 128) ? o.force_tile : 0;
        by_depth = o.group_by_depth != 0;
    }
};

kfac_options default_options()
{
    kfac_options o;
    memset(&o, 0, sizeof(o));
    o.struct_size = (int32_t)sizeof(kfac_options);
    o.fp32_products = KFAC_PRODUCTS_SPLIT_BF16;
    o.streams = 4;
    o.staging_slots = 2;
    o.correlation_form = 1;
    o.pipeline_phases = 1;
    o.early_n = 2048;
    o.target_workgroups = 128;
    o.min_k_per_split = 512;
    o.max_k_per_workgroup = 4096;
    o.recursion_leaf = 288;
    o.chunk_gflop = 48.0f;
    o.force_tile = 0;
    o.group_by_depth = 1;
    return o;
}

bool options_ok(const kfac_options *o)
{
    if (!o) return true;
    if (o->struct_size != (int32_t)sizeof(kfac_options)) return false;
    if (o->fp32_products != KFAC_PRODUCTS_SPLIT_BF16 && o->fp32_products != KFAC_PRODUCTS_FP32_MFMA) return false;
    if (o->streams < 1 || o->streams > 4 || o->staging_slots < 2 || o->staging_slots > kSlots) return false;
    if (o->early_n < 1 || o->target_workgroups < 1 || o->min_k_per_split < 32 || o->max_k_per_workgroup < 32) return false;
    if (o->recursion_leaf < 32 || o->recursion_leaf > kLeafMax) return false;
    if (!(o->chunk_gflop >= 0.0f) || !std::isfinite(o->chunk_gflop)) return false;
    if (o->force_tile != 0 && o->force_tile != 64 && o->force_tile != 128) return false;
    return true;
}

}  // namespace

struct kfac_ctx {
    hipStream_t stream;
    char *ws;
    size_t ws_bytes;
    // pinned staging ring for device tables
    char *pinned[kSlots];
    size_t pinned_bytes[kSlots];
    hipEvent_t ev[kSlots];
    bool ev_used[kSlots];
    int next_slot;
    Tunables tun{default_options()};
    // auxiliary streams (default priority) for independent chains of launches inside one call
    hipStream_t aux[3];
    hipEvent_t sync_ev[kSyncEvents];
    bool resources_ready;
    // optional per-launch timing
    bool profiling;
    std::vector<hipEvent_t> ev_pool;      // pairs: [2i] start, [2i+1] stop
    std::vector<kfac_profile_entry> prof; // one per recorded launch (ms filled at read time)
};

namespace {

// Workspace carving. With base == nullptr it only counts bytes (dry run).
struct Arena {
    char *base;
    size_t used, peak;
    explicit Arena(char *b) : base(b), used(0), peak(0) {}
    void *take(size_t bytes)
    {
        used = align_up(used, kAlign);
        char *p = base ? base + used : (char *)nullptr + used;
        used += bytes;
        peak = std::max(peak, used);
        return p;
    }
    // scratch taken after `mark` is dead once the launches that use it have been enqueued
    // (everything runs in order on one stream), so later launches may reuse it
    void release_to(size_t mark) { used = mark; }
    void *take_tail(size_t bytes) { used = peak; return take(bytes); }
};

// Host image of the device tables of one call.
struct Tables {
    std::vector<char> buf;
    size_t add(const void *data, size_t bytes)
    {
        size_t off = align_up(buf.size(), 16);
        buf.resize(off + bytes);
        if (bytes) memcpy(buf.data() + off, data, bytes);
        return off;
    }
};

enum LaunchKind { L_GEMM, L_REDUCE, L_PATCH, L_TRACE, L_COPY, L_LEAF, L_ZERO, L_BN, L_BNRED, L_PAD, L_ASSEMBLE, L_BORDER,
                  L_STALE,   // cfg: pass 0 / 1
                  L_PACK,    // cfg: 1 = unpack; dtype: 1 = bf16; p0: packed buffer
                  L_UPDATE,  // cfg: pass 0 / 1 / 2; f0: eta; f1: momentum (pass 1: f0 = eps)
                  L_LAYOUT,  // cfg: element size in bytes
                  L_BNFULL,  // cfg: pass 0 / 1 / 2; dtype: N; f0: decay; f1: lambda; p0: damp
                  L_RECORD, L_WAIT };   // stream ordering: record / wait for sync event `n` on `stream`

struct Launch {
    LaunchKind kind;
    size_t off_a, off_b;   // table offsets
    int n, total_wgs, cfg, dtype;
    float f0, f1;
    void *p0, *p1;
    double flops, bytes;   // algorithmic counts (profiling only)
    int stream;            // 0: the context's stream; 1..3: auxiliary streams (ordered by L_RECORD / L_WAIT)
};

struct Plan {
    Tables tab;
    std::vector<Launch> launches;
    void sync(LaunchKind kind, int event, int stream)
    {
        Launch L{};
        L.kind = kind; L.n = event; L.stream = stream;
        launches.push_back(L);
    }
    void set_stream(size_t first, int stream)
    {
        for (size_t q = first; q < launches.size(); ++q) launches[q].stream = stream;
    }
};

bool layer_ok(const kfac_layer &L, int *dA, int *dG, int *h, int *w)
{
    if (L.N < 1 || L.c_in < 1 || L.c_out < 1 || L.k < 1 || L.stride < 1 || L.pad < 0 || L.h_in < 1 || L.w_in < 1)
        return false;
    if (L.bias != 0 && L.bias != 1) return false;
    const long long nh = (long long)L.h_in + 2LL * L.pad - L.k, nw = (long long)L.w_in + 2LL * L.pad - L.k;
    if (nh < 0 || nw < 0) return false;
    const long long hh = nh / L.stride + 1, ww = nw / L.stride + 1;
    const long long da = (long long)L.c_in * L.k * L.k + L.bias;
    if (da > (1 << 20) || L.c_out > (1 << 20)) return false;
    if (hh * ww > (1LL << 24) || (long long)L.N * hh * ww > (1LL << 30)) return false;
    if ((long long)L.N * L.c_in * L.h_in * L.w_in > (1LL << 40)) return false;
    if (dA) *dA = (int)da;
    if (dG) *dG = L.c_out;
    if (h) *h = (int)hh;
    if (w) *w = (int)ww;
    return true;
}

// ---------------------------------------------------------------- GEMM grouping
struct GemmGroup {   // problems that go into one phase (no dependencies among them)
    std::vector<GemmProblem> probs;
};

int tile_edge(int cfg) { return cfg == 0 ? 128 : 64; }

// Rough time model (matrix-pipe cycles) of one problem under a tile configuration: the
// matrix instructions of the workgroups resident on a CU serialise per SIMD, and a lone
// wavefront per SIMD cannot hide its per-tile load/barrier latency.  Small products
// therefore prefer 64x64 tiles (4x the workgroups, a quarter of the work each).
double tile_cfg_cost(int M, int N, int K, bool sym, int cfg)
{
    const int B = cfg == 0 ? 128 : 64;
    const int slots = cfg == 0 ? 2 : 4;                 // workgroups per CU (registers / LDS)
    // cycles per wavefront per 32-wide K tile; the small tile moves twice the operand bytes
    // per flop, which costs it some efficiency on large products
    const double mfma = cfg == 0 ? 4096.0 : 1024.0 * 1.2;
    const double tm = (M + B - 1) / B, tn = (N + B - 1) / B;
    const double tiles = sym ? tm * (tm + 1) / 2 : tm * tn;
    const double per_cu = tiles / 256.0;
    const double resident = std::min<double>(slots, std::max(1.0, per_cu));
    const double rounds = std::max(1.0, per_cu / slots);
    const double ksteps = std::max(1.0, K / 32.0);
    return rounds * ksteps * std::max(mfma * resident, mfma + 700.0) + 3000.0;
}

int choose_tile_cfg(int M, int N, int K, bool sym)
{
    return tile_cfg_cost(M, N, K, sym, 0) <= tile_cfg_cost(M, N, K, sym, 1) ? 0 : 1;
}

void finish_problem(GemmProblem &P)
{
    const int B = tile_edge(P.tile_cfg);
    P.tiles_m = (P.M + B - 1) / B;
    P.tiles_n = (P.N + B - 1) / B;
    P.n_tiles = (P.flags & GEMM_SYM) ? P.tiles_m * (P.tiles_m + 1) / 2 : P.tiles_m * P.tiles_n;
    P.splits = 1;
    P.k_per_split = std::max(32, (P.K + 31) / 32 * 32);
    P.partial = nullptr;
    P.partial_rs = nullptr;
    if (P.ones == 0) P.ones = P.K;
}

// Emits the launches of one phase: per tile configuration one GEMM launch, plus one
// reduction launch if any problem was split along K (appended to `deferred` instead, if given:
// the caller then places the reductions after all the matrix launches, on a stream it chooses).
void emit_gemm_phase(Plan &plan, Arena &arena, const Tunables &tun, std::vector<GemmProblem> &probs,
                     int dtype, bool allow_split, bool phase_boost = false, std::vector<Launch> *deferred = nullptr)
{
    if (probs.empty()) return;
    // Tile configuration per problem.  When the phase as a whole keeps the GPU busy with 128x128
    // tiles, each problem takes the configuration with less padded work (the big tile moves half the
    // operand bytes per flop, worth ~15 %; up to 1.5x the work for the rectangular products of the
    // preconditioning, measured: -7 %; for the symmetric products of the factors -- 256 x 256 is 3 big
    // tiles or 10 small ones, 1.2x -- it costs the same either way); otherwise the latency model decides.
    double tile_steps128 = 0;   // 128x128 tiles times 32-wide K steps: the work of the phase
    for (auto &P : probs) {
        const double tm = (P.M + 127) / 128, tn = (P.N + 127) / 128;
        tile_steps128 += ((P.flags & GEMM_SYM) ? tm * (tm + 1) / 2 : tm * tn) * ((P.K + 31) / 32);
    }
    for (auto &P : probs) {
        const bool sym = (P.flags & GEMM_SYM) != 0;
        if (tun.force_tile) {
            P.tile_cfg = tun.force_tile == 64 ? 1 : 0;
        } else if (tile_steps128 >= 512.0 * 64) {   // every workgroup slot of the GPU busy for 64 steps
            auto work = [&](int B) {
                const double tm = (P.M + B - 1) / B, tn = (P.N + B - 1) / B;
                return (sym ? tm * (tm + 1) / 2 : tm * tn) * B * B;
            };
            P.tile_cfg = work(128) <= (phase_boost ? 1.5 : 1.15) * work(64) ? 0 : 1;
        } else {
            P.tile_cfg = choose_tile_cfg(P.M, P.N, P.K, sym);
        }
        finish_problem(P);
    }
    for (int cfg = 0; cfg < 2; ++cfg) {
        std::vector<GemmProblem> sel;
        for (auto &P : probs)
            if (P.tile_cfg == cfg) sel.push_back(P);
        if (sel.empty()) continue;
        const int B = tile_edge(cfg);
        if (allow_split) {
            // Per problem (independent of what else is in the launch, so that the workspace need of
            // a layer list does not depend on which of its inputs are present): enough splits for
            // target_wgs workgroups and at most max_k_per_wg of contraction each.
            // ... unless the launch fills the GPU twice over without that: then only max_k_per_wg splits (the
            // partial tiles of needless splits are written, read again and summed by a second launch).  The
            // workspace bound is computed with the per-problem rule, which needs the most scratch.
            long long base_wgs = 0;
            for (auto &P : sel) base_wgs += (long long)P.n_tiles * ((P.K + tun.max_k_per_wg - 1) / tun.max_k_per_wg);
            const bool launch_is_full = !tun.worst_case_splits && base_wgs >= (cfg == 0 ? 1024 : 2048);
            auto splits_for = [&](const GemmProblem &P, int boost, int *kps_out) {
                const int want = std::max(boost, launch_is_full ? 1 : (tun.target_wgs + P.n_tiles - 1) / P.n_tiles);
                int splits = std::max((P.K + tun.max_k_per_wg - 1) / tun.max_k_per_wg,
                                      std::min(want, P.K / tun.min_k_per_split));
                int kps = std::max(32, (P.K + 31) / 32 * 32);
                if (splits > 1) {
                    kps = ((P.K + splits - 1) / splits + 31) / 32 * 32;
                    splits = (P.K + kps - 1) / kps;
                }
                *kps_out = kps;
                return std::max(1, splits);
            };
            // A heavy phase with only a few rounds of workgroups (a CU holds two 128x128 or four
            // 64x64 workgroups) loses a large part of its last round: 1026 equal tiles on 512 slots
            // take 3 rounds, not 2.004.  Splitting every problem `boost` times further shortens the
            // rounds; the boost with the shortest modelled makespan wins (each extra split charged
            // 2 % for the partial tiles and their reduction).  Only for phases whose problem set is
            // fixed by the layer list.
            int boost = 1;
            if (phase_boost) {
                const double slots = cfg == 0 ? 512.0 : 1024.0;
                double ksteps = 0;
                for (auto &P : sel) ksteps += (double)P.n_tiles * ((P.K + 31) / 32);
                if (ksteps >= slots * 24) {
                    double best = 0;
                    for (int cand = 1; cand <= 8; ++cand) {
                        double work = 0, longest = 0;
                        for (auto &P : sel) {
                            int kps;
                            const int sp = splits_for(P, cand, &kps);
                            const double len = kps / 32 + 6.0;   // K steps plus the fixed part of a workgroup
                            work += (double)P.n_tiles * sp * len;
                            longest = std::max(longest, len);
                        }
                        const double makespan = std::ceil(work / (longest * slots)) * longest * (1.0 + 0.02 * (cand - 1));
                        if (cand == 1 || makespan < best) { best = makespan; boost = cand; }
                    }
                }
            }
            for (auto &P : sel) {
                int kps;
                const int splits = splits_for(P, boost, &kps);
                if (splits > 1) {
                    P.splits = splits;
                    P.k_per_split = kps;
                    P.partial = (float *)arena.take((size_t)P.n_tiles * splits * B * B * sizeof(float));
                    if (P.flags & GEMM_BORDER)
                        P.partial_rs = (float *)arena.take((size_t)P.tiles_m * splits * B * sizeof(float));
                }
            }
        }
        // longest workgroups first
        std::stable_sort(sel.begin(), sel.end(), [](const GemmProblem &x, const GemmProblem &y) {
            return std::min(x.K, x.k_per_split) > std::min(y.K, y.k_per_split);
        });
        std::vector<int> start(sel.size() + 1, 0), rstart(sel.size() + 1, 0);
        bool any_split = false;
        for (size_t i = 0; i < sel.size(); ++i) {
            start[i + 1] = start[i] + ((sel[i].n_tiles * sel[i].splits + 7) & ~7);   // XCD-aligned
            rstart[i + 1] = rstart[i] + (sel[i].splits > 1 ? sel[i].n_tiles * (B / 32) : 0);
            any_split |= sel[i].splits > 1;
        }
        Launch L{};
        L.kind = L_GEMM;
        for (auto &P : sel)
            if (P.flags & GEMM_SYM) {
                const double d = P.M + ((P.flags & GEMM_BORDER) ? 1.0 : 0.0);
                L.flops += (double)P.K * d * (d + 1.0);
            } else {
                L.flops += 2.0 * P.M * (double)P.N * P.K;
            }
        L.off_a = plan.tab.add(sel.data(), sel.size() * sizeof(GemmProblem));
        L.off_b = plan.tab.add(start.data(), start.size() * sizeof(int));
        L.n = (int)sel.size();
        L.total_wgs = start.back();
        L.cfg = cfg;
        L.dtype = (dtype == 0 && tun.split) ? 2 : dtype;
        plan.launches.push_back(L);
        if (any_split) {
            Launch R{};
            R.kind = L_REDUCE;
            R.off_a = L.off_a;
            R.off_b = plan.tab.add(rstart.data(), rstart.size() * sizeof(int));
            R.n = (int)sel.size();
            R.total_wgs = rstart.back();
            for (auto &P : sel)
                if (P.splits > 1) R.bytes += 4.0 * P.n_tiles * B * B * (P.splits + 1.0);   // partial tiles read, the sum written
            if (deferred) deferred->push_back(R);
            else plan.launches.push_back(R);
        }
    }
}

Operand plain_operand(const float *base, long long ld, int rows, int K)
{
    Operand o{};
    o.base = base;
    o.row_stride = ld;
    o.batch_stride = 0;
    o.rows = rows;
    o.hw = std::max(K, 1) + 64;   // one run covers the whole contraction
    return o;
}

// ---------------------------------------------------------------- stats planner
struct StatsArgs {
    int n_layers;
    const kfac_layer *L;
    kfac_dtype in;
    const void *const *act;
    const void *const *grad_out;
    float decay;
    int g_spatial_mean;
    float *const *A_ema;
    float *const *G_ema;
    int nhwc = 0;   // 1: act is [N, H, W, C_in] and grad_out [N, h, w, C_out]
};

// Workgroups of one patch / repack job.
int patch_job_wgs(const PatchJob &J)
{
    const int hw = J.h * J.w;
    if (J.flat) return J.c_in * ((J.N * hw + 255) / 256);
    return ((J.N * J.c_in + 3) / 4) * ((hw + 1023) / 1024);
}

PatchJob make_patch_job(const void *src, void *dst, long long ld, int N, int c, int k, int stride, int pad,
                        int h_in, int w_in, int h, int w, int esize)
{
    PatchJob J{};
    J.src = src; J.dst = dst; J.ld = ld;
    J.N = N; J.c_in = c; J.k = k; J.stride = stride; J.pad = pad;
    J.h_in = h_in; J.w_in = w_in; J.h = h; J.w = w;
    J.esize = esize;
    J.flat = (k == 1 && stride == 1 && pad == 0 && h * w < 64) ? 1 : 0;
    J.magic_w = (h * w < 65536 && w > 1) ? (unsigned)((1ULL << 32) / (unsigned)w + 1ULL) : 0u;
    return J;
}

// `subset` (or null for all): the layers of `a` to build factors for.
// Where the parts of one factor phase run when it is spread over streams: the operand
// rewrites (patch extraction, zero padding) ahead of the matrix launches on `pre_stream`, the
// matrix launches on the context's stream, what follows them (split-K reductions, assembly of
// the correlation form) on `post_stream`, which is where the phase's factors are complete.
// A stream of 0 keeps that part on the context's stream.
struct StatsSplit {
    int pre_stream, ev_pre;     // event recorded when the rewrites are done
    int post_stream, ev_gemm;   // event recorded when the matrix launches are done
    int gemm_chunks;            // the matrix launches are cut into this many successive parts (<= 1: not)
};

void plan_stats(Plan &plan, Arena &arena, const Tunables &tun, const StatsArgs &a, bool dry,
                const std::vector<int> *subset = nullptr, const StatsSplit *split = nullptr)
{
    const int esize = a.in == KFAC_BF16 ? 2 : 4;
    // a thread loads 16-byte chunks: 4 fp32 (element alignment is enough) or 8 bf16 (16-byte aligned)
    const int chunk = a.in == KFAC_BF16 ? 8 : 4;
    const size_t chunk_align = a.in == KFAC_BF16 ? 16 : 4;
    std::vector<PatchJob> pjobs;
    std::vector<PadJob> padjobs;
    std::vector<PadJobBF16> padbfjobs;
    int padbf_wgs = 0;
    std::vector<AssembleJob> asmjobs;
    std::vector<GemmProblem> probs;
    std::vector<GemmProblem> tprobs;   // products of operands stored transposed (NHWC tensors in place): launches of their own
    std::vector<LayoutJob> ljobs;      // NHWC tensors whose layer needs the NCHW order: converted into scratch first
    long long layout_wgs = 0;
    double layout_bytes = 0;
    // An NHWC tensor is contracted in place by the transposed loader if it belongs to a pointwise layer and its
    // channel count is a whole number of 16-byte chunks (fp32: in the three-plane product mode only; bf16: base
    // 16-byte aligned); everything else is first brought into NCHW order (the kernel of kfac_nhwc_to_nchw) and
    // then treated as usual.
    auto to_nchw = [&](const void *src, int N, int c, int hw_in) -> const void * {
        void *dst = arena.take((size_t)N * c * hw_in * esize);
        LayoutJob J{};
        J.src = src; J.dst = dst;
        J.N = N; J.C = c; J.HW = hw_in;
        J.tiles_c = (c + 63) / 64;
        J.tiles_hw = (hw_in + 63) / 64;
        J.wg_start = (int)layout_wgs;
        layout_wgs += (long long)N * J.tiles_c * J.tiles_hw;
        layout_bytes += 2.0 * (double)N * c * hw_in * esize;
        ljobs.push_back(J);
        return dry ? nullptr : dst;
    };
    int patch_wgs = 0, pad_wgs = 0, asm_wgs = 0;
    double patch_bytes = 0, pad_bytes = 0, asm_bytes = 0;
    // An NCHW tensor [N, c, hw] is contracted in place when its runs are whole chunks; otherwise (and for every k > 1 / strided / padded layer) it is first rewritten
    // as [c k^2][ld] with the contraction index contiguous.
    // (*K_out: the length of the contraction over this operand)
    auto operand_for = [&](const void *src, int N, int c, int k, int stride, int pad, int h_in, int w_in, int h,
                           int w, int *K_out) {
        const int hw = h * w, K = N * hw, d0 = c * k * k;
        *K_out = K;
        Operand op{};
        const bool pointwise = k == 1 && stride == 1 && pad == 0;
        if (a.nhwc) {
            const bool in_place = a.in == KFAC_F32 ? (tun.split && c % 4 == 0)
                                                   : (c % 8 == 0 && (dry || ((uintptr_t)src % 16) == 0));
            if (pointwise && in_place) {
                op.base = src;
                op.row_stride = c;     // from one position to the next
                op.batch_stride = 0;
                op.rows = c;
                op.hw = K + 64;
                op.trans = 1;
                return op;
            }
            src = to_nchw(src, N, c, h_in * w_in);
        }
        const bool direct = pointwise && hw % chunk == 0 && (dry || ((uintptr_t)src % chunk_align) == 0);
        // bf16 runs of 8q + 4 (14 x 14 planes): in place as well, the last chunk of a run in two halves
        const bool direct_tail = pointwise && !direct && a.in == KFAC_BF16 && hw % 8 == 4 && hw >= 12 &&
                                 (dry || ((uintptr_t)src % 8) == 0);
        if (direct || direct_tail) {
            op.base = src;
            op.row_stride = hw;
            op.batch_stride = (long long)c * hw;
            op.rows = d0;
            op.hw = direct ? hw : hw + 4;
            op.tail = direct ? 0 : 4;
            *K_out = N * op.hw;
        } else {
            const long long ld = align_up((size_t)K, 32);
            void *P = arena.take((size_t)d0 * ld * esize);
            PatchJob J = make_patch_job(src, P, ld, N, c, k, stride, pad, h_in, w_in, h, w, esize);
            J.wg_start = patch_wgs;
            patch_wgs += patch_job_wgs(J);
            patch_bytes += (double)esize * ((double)N * c * h_in * w_in + (double)d0 * K);
            pjobs.push_back(J);
            op.base = P;
            op.row_stride = ld;
            op.batch_stride = 0;
            op.rows = d0;
            op.hw = K + 64;
        }
        return op;
    };
    const int n_sel = subset ? (int)subset->size() : a.n_layers;
    for (int q = 0; q < n_sel; ++q) {
        const int l = subset ? (*subset)[q] : q;
        const kfac_layer &Ly = a.L[l];
        int dA, dG, h, w;
        layer_ok(Ly, &dA, &dG, &h, &w);
        const int hw = h * w;
        const int K = Ly.N * hw;
        const bool want_A = dry || (a.act && a.act[l]);
        const bool want_G = dry || (a.grad_out && a.grad_out[l]);
        // 3x3 / stride 1 / pad 1: 13 displaced correlations of the zero-padded image instead of the
        // 81 C^2 products of the patch Gram matrix, if the padding does not eat the gain (26 PP < 81 hw
        // flops-wise).  fp32: at least two zero rows above and two zero columns left of every image, a
        // few more if that is what makes the padded plane a whole number of 16-byte chunks.  bf16: the
        // padded width a multiple of 8, so that a row displacement keeps 16-byte alignment (the column
        // displacements come from shifted copies, see PadJobBF16).
        const bool bf = a.in == KFAC_BF16;
        int Hp = 0, Wp = 0;
        if (bf) { Hp = h + 2; Wp = (int)align_up((size_t)w + 2, 8); }
        else
            for (int eh = 2; eh <= 5; ++eh)
                for (int ew = 2; ew <= 5; ++ew)
                    if (((h + eh) * (w + ew)) % 4 == 0 && (Hp == 0 || (h + eh) * (w + ew) < Hp * Wp)) { Hp = h + eh; Wp = w + ew; }
        const bool corr = tun.corr && Ly.k == 3 && Ly.stride == 1 && Ly.pad == 1 && h >= 3 && w >= 3 &&
                          2 * Hp * Wp <= 5 * hw;
        if (want_A && corr) {
            const int C = Ly.c_in, N = Ly.N, PP = Hp * Wp;
            const void *act_l = dry ? nullptr : a.act[l];
            if (a.nhwc) act_l = to_nchw(act_l, N, C, h * w);
            const int lal = bf ? 8 : 4;   // line lengths in whole 16-byte chunks
            const int Lw = (int)align_up((size_t)w + 2, lal), Lh = (int)align_up((size_t)h + 2, lal);
            // operands of the contractions: the image, the image displaced by (dy, dx), border lines shifted by d, corners
            std::function<Operand(int, int)> image_op;
            std::function<Operand(int, int)> row_op, col_op;   // (which, shift)
            std::function<Operand(int)> corner_op;
            int corner_K = N;
            if (!bf) {
                PadJob J{};
                J.src = (const float *)act_l;
                J.front_slack = (int)align_up((size_t)2 * Wp + 2, 4);
                J.padded_floats = (long long)J.front_slack + (long long)N * C * PP + (long long)align_up((size_t)2 * Wp + 2, 4) + 4;
                J.padded = (float *)arena.take((size_t)J.padded_floats * sizeof(float));
                J.rows = (float *)arena.take(((size_t)2 * C * N * Lw + 4) * sizeof(float));
                J.cols = (float *)arena.take(((size_t)2 * C * N * Lh + 4) * sizeof(float));
                J.corners = (float *)arena.take(((size_t)4 * C * N + 4) * sizeof(float));
                J.N = N; J.C = C; J.H = h; J.W = w; J.Hp = Hp; J.Wp = Wp; J.Lw = Lw; J.Lh = Lh;
                J.wg_start = pad_wgs;
                const long long threads = J.padded_floats / 4 + (2LL * C * N * Lw + 4) + (2LL * C * N * Lh + 4) + 4LL * C * N;
                pad_wgs += (int)((threads + 255) / 256);
                pad_bytes += 4.0 * ((double)N * C * hw + (double)J.padded_floats);
                padjobs.push_back(J);
                image_op = [=](int dy, int dx) {
                    Operand o{};
                    o.base = J.padded + J.front_slack + dy * Wp + dx;
                    o.row_stride = PP; o.batch_stride = (long long)C * PP; o.rows = C; o.hw = PP;
                    return o;
                };
                row_op = [=](int which, int d) { return plain_operand(J.rows + (size_t)which * C * N * Lw + d, (long long)N * Lw, C, N * Lw); };
                col_op = [=](int which, int d) { return plain_operand(J.cols + (size_t)which * C * N * Lh + d, (long long)N * Lh, C, N * Lh); };
                corner_op = [=](int wc) { return plain_operand(J.corners + (size_t)wc * C * N, N, C, N); };
            } else {
                PadJobBF16 J{};
                const int Ln = (int)align_up((size_t)N, 8);
                J.src = (const unsigned short *)act_l;
                J.front_slack = (int)align_up((size_t)2 * Wp + 2, 8);
                J.copy_elems = (long long)J.front_slack + (long long)N * C * PP + (long long)align_up((size_t)2 * Wp + 2, 8) + 8;
                J.rows_elems = (long long)align_up((size_t)2 * C * N * Lw + 8, 8);
                J.cols_elems = (long long)align_up((size_t)2 * C * N * Lh + 8, 8);
                J.padded = (unsigned short *)arena.take((size_t)5 * J.copy_elems * 2);
                J.rows = (unsigned short *)arena.take((size_t)3 * J.rows_elems * 2);
                J.cols = (unsigned short *)arena.take((size_t)3 * J.cols_elems * 2);
                J.corners = (unsigned short *)arena.take((size_t)4 * C * Ln * 2);
                J.N = N; J.C = C; J.H = h; J.W = w; J.Hp = Hp; J.Wp = Wp; J.Lw = Lw; J.Lh = Lh; J.Ln = Ln;
                J.wg_start = padbf_wgs;
                const long long threads = J.copy_elems / 8 + 3 * J.rows_elems + 3 * J.cols_elems + 4LL * C * Ln;
                padbf_wgs += (int)((threads + 255) / 256);
                pad_bytes += 2.0 * ((double)N * C * hw + 5.0 * (double)J.copy_elems);
                padbfjobs.push_back(J);
                auto plain16 = [](const unsigned short *base, long long ld, int rows, int K) {
                    Operand o{};
                    o.base = base; o.row_stride = ld; o.batch_stride = 0; o.rows = rows; o.hw = std::max(K, 1) + 64;
                    return o;
                };
                image_op = [=](int dy, int dx) {
                    Operand o{};
                    o.base = J.padded + (long long)(dx + 2) * J.copy_elems + J.front_slack + dy * Wp;
                    o.row_stride = PP; o.batch_stride = (long long)C * PP; o.rows = C; o.hw = PP;
                    return o;
                };
                row_op = [=](int which, int d) { return plain16(J.rows + (long long)d * J.rows_elems + (size_t)which * C * N * Lw, (long long)N * Lw, C, N * Lw); };
                col_op = [=](int which, int d) { return plain16(J.cols + (long long)d * J.cols_elems + (size_t)which * C * N * Lh, (long long)N * Lh, C, N * Lh); };
                corner_op = [=](int wc) { return plain16(J.corners + (size_t)wc * C * Ln, Ln, C, Ln); };
                corner_K = Ln;
            }

            AssembleJob S{};
            S.A = dry ? nullptr : a.A_ema[l];
            S.ldA = dA; S.C = C; S.bias = Ly.bias;
            S.alpha = (float)((1.0 - (double)a.decay) / ((double)N * (double)hw));
            S.beta = a.decay;
            S.count = (float)((double)N * (double)hw);
            S.wg_start = asm_wgs;
            asm_wgs += dA;   // one workgroup per row of A
            asm_bytes += 4.0 * dA * dA * (a.decay != 0.f ? 2.0 : 1.0) + 4.0 * 50.0 * C * C;   // A (read too under a running average) and about 50 C x C Gram matrices / transposed copies
            // one Gram matrix per contraction; those with displacement 0 are symmetric and carry the row sums
            auto gram = [&](const Operand &oa, const Operand &ob, int K, bool zero_shift, const float **out,
                            const float **out_t, int *ld) {
                GemmProblem P{};
                P.a = oa; P.b = ob;
                const int ldc = zero_shift ? C + 1 : C;
                P.C = (float *)arena.take((size_t)ldc * ldc * sizeof(float));
                P.ldc = ldc;
                P.Ct = zero_shift ? nullptr : (float *)arena.take((size_t)ldc * ldc * sizeof(float));
                P.ldct = ldc;
                P.M = C; P.N = C; P.K = K;
                P.flags = zero_shift ? (GEMM_SYM | GEMM_BORDER) : 0;
                P.alpha = 1.f; P.beta = 0.f;
                P.tile_cfg = choose_tile_cfg(C, C, K, zero_shift);
                finish_problem(P);
                probs.push_back(P);
                *out = P.C; *ld = ldc;
                if (out_t) *out_t = zero_shift ? P.C : P.Ct;
            };
            const Operand img = image_op(0, 0);
            for (int slot = 0; slot < 13; ++slot) {
                const int dy = slot < 3 ? 0 : (slot - 3) / 5 + 1, dx = slot < 3 ? slot : (slot - 3) % 5 - 2;
                gram(img, image_op(dy, dx), N * PP, slot == 0, &S.full[slot], &S.full_t[slot], &S.ld_full[slot]);
            }
            for (int which = 0; which < 2; ++which)
                for (int d = 0; d < 3; ++d) {
                    gram(row_op(which, 0), row_op(which, d), N * Lw, d == 0, &S.rows[which][d], &S.rows_t[which][d], &S.ld_rows[which][d]);
                    gram(col_op(which, 0), col_op(which, d), N * Lh, d == 0, &S.cols[which][d], &S.cols_t[which][d], &S.ld_cols[which][d]);
                }
            for (int wc = 0; wc < 4; ++wc) {
                int ld = 0;
                gram(corner_op(wc), corner_op(wc), corner_K, true, &S.corners[wc], nullptr, &ld);
                S.ld_corner = ld;
            }
            asmjobs.push_back(S);
        } else if (want_A) {
            int Kop = K;
            Operand op = operand_for(dry ? nullptr : a.act[l], Ly.N, Ly.c_in, Ly.k, Ly.stride, Ly.pad, Ly.h_in,
                                     Ly.w_in, h, w, &Kop);
            // the bias row of the patch matrix is not multiplied out: the border of A comes
            // from row sums (GEMM_BORDER), which keeps c_in k^2 a whole number of tiles
            GemmProblem P{};
            P.a = op; P.b = op;
            P.C = dry ? nullptr : a.A_ema[l];
            P.Ct = nullptr;
            P.ldc = dA; P.ldct = 0;
            P.M = op.rows; P.N = op.rows; P.K = Kop;
            P.ones = K;   // the bias row has a one per real position (Kop counts the zero tail of bf16 runs as well)
            P.flags = GEMM_SYM | (Ly.bias ? GEMM_BORDER : 0);
            P.tile_cfg = choose_tile_cfg(P.M, P.N, K, true);
            P.alpha = (float)((1.0 - (double)a.decay) / ((double)Ly.N * (double)hw));
            P.beta = a.decay;
            if (op.trans) P.flags |= GEMM_TRANS;
            finish_problem(P);
            (op.trans ? tprobs : probs).push_back(P);
        }
        if (want_G) {
            int Kop = K;
            Operand op = operand_for(dry ? nullptr : a.grad_out[l], Ly.N, Ly.c_out, 1, 1, 0, h, w, h, w, &Kop);
            GemmProblem P{};
            P.a = op; P.b = op;
            P.C = dry ? nullptr : a.G_ema[l];
            P.ldc = dG;
            P.M = dG; P.N = dG; P.K = Kop;
            P.flags = GEMM_SYM;
            P.tile_cfg = choose_tile_cfg(dG, dG, K, true);
            double scale = 1.0 / (double)Ly.N;
            if (a.g_spatial_mean) scale /= (double)hw;
            P.alpha = (float)((1.0 - (double)a.decay) * scale);
            P.beta = a.decay;
            if (op.trans) P.flags |= GEMM_TRANS;
            finish_problem(P);
            (op.trans ? tprobs : probs).push_back(P);
        }
    }
    const size_t first_pre = plan.launches.size();
    if (!ljobs.empty()) {
        Launch L{};
        L.kind = L_LAYOUT;
        L.off_a = plan.tab.add(ljobs.data(), ljobs.size() * sizeof(LayoutJob));
        L.n = (int)ljobs.size();
        L.total_wgs = (int)layout_wgs;
        L.cfg = esize;
        L.bytes = layout_bytes;
        plan.launches.push_back(L);
    }
    if (!pjobs.empty()) {
        Launch L{};
        L.kind = L_PATCH;
        L.off_a = plan.tab.add(pjobs.data(), pjobs.size() * sizeof(PatchJob));
        L.n = (int)pjobs.size();
        L.total_wgs = patch_wgs;
        L.bytes = patch_bytes;
        plan.launches.push_back(L);
    }
    if (!padjobs.empty()) {
        Launch L{};
        L.kind = L_PAD;
        L.off_a = plan.tab.add(padjobs.data(), padjobs.size() * sizeof(PadJob));
        L.n = (int)padjobs.size();
        L.total_wgs = pad_wgs;
        L.bytes = pad_bytes;
        plan.launches.push_back(L);
    }
    if (!padbfjobs.empty()) {
        Launch L{};
        L.kind = L_PAD;
        L.off_a = plan.tab.add(padbfjobs.data(), padbfjobs.size() * sizeof(PadJobBF16));
        L.n = (int)padbfjobs.size();
        L.total_wgs = padbf_wgs;
        L.cfg = 1;   // the bf16 form
        L.bytes = pad_bytes;
        plan.launches.push_back(L);
    }
    if (split && split->pre_stream > 0 && plan.launches.size() > first_pre) {
        plan.set_stream(first_pre, split->pre_stream);
        plan.sync(L_RECORD, split->ev_pre, split->pre_stream);
        plan.sync(L_WAIT, split->ev_pre, 0);
    }
    const int post = split ? split->post_stream : 0;
    std::vector<Launch> reductions;
    {
        const int nchunk = split ? std::max(1, split->gemm_chunks) : 1;
        if (nchunk <= 1) {
            emit_gemm_phase(plan, arena, tun, probs, a.in == KFAC_BF16 ? 1 : 0, true, false, post > 0 ? &reductions : nullptr);
        } else {
            // chunks of similar work (largest problems first, each to the lightest chunk)
            std::vector<size_t> order(probs.size());
            for (size_t i = 0; i < order.size(); ++i) order[i] = i;
            auto work = [&](const GemmProblem &P) { return (double)P.M * P.N * P.K; };
            std::stable_sort(order.begin(), order.end(), [&](size_t x, size_t y) { return work(probs[x]) > work(probs[y]); });
            std::vector<std::vector<GemmProblem>> chunks(nchunk);
            std::vector<double> load(nchunk, 0.0);
            for (size_t i : order) {
                int g = 0;
                for (int q = 1; q < nchunk; ++q) if (load[q] < load[g]) g = q;
                chunks[g].push_back(probs[i]);
                load[g] += work(probs[i]);
            }
            for (auto &c : chunks)
                emit_gemm_phase(plan, arena, tun, c, a.in == KFAC_BF16 ? 1 : 0, true, false, post > 0 ? &reductions : nullptr);
        }
        emit_gemm_phase(plan, arena, tun, tprobs, a.in == KFAC_BF16 ? 4 : 3, true, false, post > 0 ? &reductions : nullptr);
    }
    if (post > 0) {
        plan.sync(L_RECORD, split->ev_gemm, 0);
        plan.sync(L_WAIT, split->ev_gemm, post);
        for (auto &R : reductions) {
            R.stream = post;
            plan.launches.push_back(R);
        }
    }
    if (!asmjobs.empty()) {
        Launch L{};
        L.kind = L_ASSEMBLE;
        L.off_a = plan.tab.add(asmjobs.data(), asmjobs.size() * sizeof(AssembleJob));
        L.n = (int)asmjobs.size();
        L.total_wgs = asm_wgs;
        L.bytes = asm_bytes;
        L.stream = post;
        plan.launches.push_back(L);
    }
}

// ---------------------------------------------------------------- inversion planner
struct InvMatrix {
    const float *src;
    float *dst;
    int n, damp_idx, info_idx;
    bool bias;   // an A factor whose last row/column is the bias border
};

enum OpKind { OP_LEAF, OP_GEMM };
struct InvOp {
    int level;
    OpKind kind;
    LeafJob leaf;
    GemmProblem gemm;
};

int leaf_class(int n)
{
    for (int c = 0; c < kNumLeafClasses; ++c)
        if (n <= 32 * kLeafClasses[c]) return c;
    return -1;
}

int split_point(int n)
{
    int n1 = ((n / 2) + 16) / 32 * 32;
    n1 = std::max(32, std::min(n1, n - 1));
    return n1;
}

// Recursive 2x2 block inversion through the Schur complement, in place in X (leading
// dimension ld) on the diagonal block starting at `o` of size n.  With X = [A11 A12; A21 A22]:
//   X11 <- A11^-1                                  (recursion)
//   Y   = A21 X11,  W = Y^T                        (GEMM, both copies kept in scratch)
//   X22 <- A22 - Y A21^T  = S                      (GEMM, symmetric)
//   X22 <- S^-1                                    (recursion)
//   X12 <- -W X22,  X21 <- X12^T                   (GEMM + transposed copy)
//   X11 <- X11 - X12 W^T                           (GEMM, symmetric)
// Returns the first level at which the block's inverse is complete.
int build_inverse(std::vector<InvOp> &ops, Arena &arena, float *X, long long ld, int o, int n, int level,
                  int info_idx, int rec_leaf)
{
    if (n <= rec_leaf) {
        InvOp op{};
        op.level = level;
        op.kind = OP_LEAF;
        float *v = X + (long long)o * ld + o;
        op.leaf.src = v; op.leaf.dst = v;
        op.leaf.lds = ld; op.leaf.ldd = ld;
        op.leaf.n = n;
        op.leaf.damp_idx = -1;
        op.leaf.info_idx = info_idx;
        op.leaf.pivot_base = o;
        ops.push_back(op);
        return level + 1;
    }
    const int n1 = split_point(n), n2 = n - n1;
    float *X11 = X + (long long)o * ld + o;
    float *X12 = X11 + n1;
    float *X21 = X11 + (long long)n1 * ld;
    float *X22 = X21 + n1;
    const long long ldy = align_up((size_t)n1, 4), ldw = align_up((size_t)n2, 4);
    float *Y = (float *)arena.take((size_t)n2 * ldy * sizeof(float));
    float *W = (float *)arena.take((size_t)n1 * ldw * sizeof(float));

    const int l1 = build_inverse(ops, arena, X, ld, o, n1, level, info_idx, rec_leaf);
    {
        InvOp op{};
        op.level = l1; op.kind = OP_GEMM;
        GemmProblem &P = op.gemm;
        P.a = plain_operand(X21, ld, n2, n1);
        P.b = plain_operand(X11, ld, n1, n1);
        P.C = Y; P.ldc = ldy; P.Ct = W; P.ldct = ldw;
        P.M = n2; P.N = n1; P.K = n1; P.flags = 0;
        P.alpha = 1.f; P.beta = 0.f;
        P.tile_cfg = choose_tile_cfg(P.M, P.N, P.K, (P.flags & GEMM_SYM) != 0);
        finish_problem(P);
        ops.push_back(op);
    }
    {
        InvOp op{};
        op.level = l1 + 1; op.kind = OP_GEMM;
        GemmProblem &P = op.gemm;
        P.a = plain_operand(Y, ldy, n2, n1);
        P.b = plain_operand(X21, ld, n2, n1);
        P.C = X22; P.ldc = ld; P.Ct = nullptr;
        P.M = n2; P.N = n2; P.K = n1; P.flags = GEMM_SYM;
        P.alpha = -1.f; P.beta = 1.f;
        P.tile_cfg = choose_tile_cfg(P.M, P.N, P.K, (P.flags & GEMM_SYM) != 0);
        finish_problem(P);
        ops.push_back(op);
    }
    const int l2 = build_inverse(ops, arena, X, ld, o + n1, n2, l1 + 2, info_idx, rec_leaf);
    {
        InvOp op{};
        op.level = l2; op.kind = OP_GEMM;
        GemmProblem &P = op.gemm;
        P.a = plain_operand(W, ldw, n1, n2);
        P.b = plain_operand(X22, ld, n2, n2);
        P.C = X12; P.ldc = ld; P.Ct = X21; P.ldct = ld;
        P.M = n1; P.N = n2; P.K = n2; P.flags = 0;
        P.alpha = -1.f; P.beta = 0.f;
        P.tile_cfg = choose_tile_cfg(P.M, P.N, P.K, (P.flags & GEMM_SYM) != 0);
        finish_problem(P);
        ops.push_back(op);
    }
    {
        InvOp op{};
        op.level = l2 + 1; op.kind = OP_GEMM;
        GemmProblem &P = op.gemm;
        P.a = plain_operand(X12, ld, n1, n2);
        P.b = plain_operand(W, ldw, n1, n2);
        P.C = X11; P.ldc = ld; P.Ct = nullptr;
        P.M = n1; P.N = n1; P.K = n2; P.flags = GEMM_SYM;
        P.alpha = -1.f; P.beta = 1.f;
        P.tile_cfg = choose_tile_cfg(P.M, P.N, P.K, (P.flags & GEMM_SYM) != 0);
        finish_problem(P);
        ops.push_back(op);
    }
    return l2 + 2;
}

struct InvertArgs {
    int n_layers;
    const kfac_layer *L;
    const float *const *A_ema;
    const float *const *G_ema;
    float gamma;
    float *const *A_inv;
    float *const *G_inv;
    float *pi_out;
    int32_t *info;
};

// Inversion of a list of damped SPD matrices as one chain of launches: the damped copies, then
// the recursion of every matrix with the launches of equal depth merged, then the bias borders.
// damp: device array the matrices' damp_idx point into; info: device array for info_idx or null.
void plan_invert_mats(Plan &plan, Arena &arena, const Tunables &tun, const std::vector<InvMatrix> &mats,
                      float *damp, int32_t *info)
{
    std::vector<CopyJob> cjobs;
    std::vector<BorderJob> bjobs;
    int copy_wgs = 0, border_wgs = 0;
    double copy_bytes = 0, border_bytes = 0;
    std::vector<InvOp> ops;
    for (const InvMatrix &m : mats) {
        if (m.n <= kLeafMax) {
            InvOp op{};
            op.level = 0; op.kind = OP_LEAF;
            op.leaf.src = m.src; op.leaf.dst = m.dst;
            op.leaf.lds = m.n; op.leaf.ldd = m.n;
            op.leaf.n = m.n;
            op.leaf.damp_idx = m.damp_idx;
            op.leaf.info_idx = m.info_idx;
            op.leaf.pivot_base = 0;
            ops.push_back(op);
        } else {
            // The bias border (c_in k^2 + 1) would make every block of the recursion one row larger
            // than a whole number of tiles.  It is eliminated first instead, inside the copy (Schur
            // complement of the 1x1 corner), and put back into the finished inverse at the end.
            const int core = m.bias ? m.n - 1 : m.n;
            CopyJob C{};
            C.src = m.src; C.dst = m.dst;
            C.lds = m.n; C.ldd = m.n; C.n = core;
            C.damp_idx = m.damp_idx;
            C.border = m.bias ? 1 : 0;
            C.wg_start = copy_wgs;
            copy_wgs += (core + 7) / 8;
            copy_bytes += 8.0 * core * core;   // every element read once and written once
            cjobs.push_back(C);
            build_inverse(ops, arena, m.dst, m.n, 0, core, 0, m.info_idx, tun.rec_leaf);
            if (m.bias) {
                BorderJob B{};
                B.src = m.src; B.X = m.dst;
                B.lds = m.n; B.ldx = m.n; B.n = core;
                B.damp_idx = m.damp_idx; B.info_idx = m.info_idx;
                B.wg_start = border_wgs;
                border_wgs += (core + 3) / 4;
                border_bytes += 4.0 * core * core;   // pass 0 reads the core inverse once
                bjobs.push_back(B);
            }
        }
    }
    if (!cjobs.empty()) {
        Launch C{};
        C.kind = L_COPY;
        C.off_a = plan.tab.add(cjobs.data(), cjobs.size() * sizeof(CopyJob));
        C.n = (int)cjobs.size();
        C.total_wgs = copy_wgs;
        C.p0 = damp;
        C.bytes = copy_bytes;
        plan.launches.push_back(C);
    }
    int max_level = -1;
    for (auto &op : ops) max_level = std::max(max_level, op.level);
    for (int lv = 0; lv <= max_level; ++lv) {
        for (int c = 0; c < kNumLeafClasses; ++c) {
            std::vector<LeafJob> lj;
            for (auto &op : ops)
                if (op.level == lv && op.kind == OP_LEAF && leaf_class(op.leaf.n) == c) lj.push_back(op.leaf);
            if (lj.empty()) continue;
            Launch Lf{};
            Lf.kind = L_LEAF;
            Lf.off_a = plan.tab.add(lj.data(), lj.size() * sizeof(LeafJob));
            Lf.n = (int)lj.size();
            Lf.cfg = c;
            Lf.p0 = damp;
            Lf.p1 = info;
            plan.launches.push_back(Lf);
        }
        std::vector<GemmProblem> gp;
        for (auto &op : ops)
            if (op.level == lv && op.kind == OP_GEMM) gp.push_back(op.gemm);
        // split-K scratch of one level is dead once the level's launches are enqueued (in order)
        const size_t mark = arena.used;
        emit_gemm_phase(plan, arena, tun, gp, 0, true, true);
        arena.release_to(mark);
    }
    if (!bjobs.empty()) {
        const size_t off = plan.tab.add(bjobs.data(), bjobs.size() * sizeof(BorderJob));
        for (int pass = 0; pass < 2; ++pass) {
            Launch B{};
            B.kind = L_BORDER;
            B.off_a = off;
            B.n = (int)bjobs.size();
            B.total_wgs = border_wgs;
            B.cfg = pass;
            B.p0 = damp;
            B.p1 = info;
            B.bytes = pass == 0 ? border_bytes : 0.0;
            plan.launches.push_back(B);
        }
    }
}

// Inversion of both factors of the layers `ids` as one chain of launches on `stream`:
// traces / damping, the damped copies, then the recursion of every matrix with the launches
// of equal depth merged.  damp: [3 * n_layers] floats shared by all groups of the call.
void plan_invert_group(Plan &plan, Arena &arena, const Tunables &tun, const InvertArgs &a, bool dry,
                       const std::vector<int> &ids, float *damp, int stream)
{
    if (ids.empty()) return;
    const size_t first_launch = plan.launches.size();
    std::vector<TraceJob> tjobs;
    std::vector<InvMatrix> mats;
    for (int l : ids) {
        int dA, dG;
        layer_ok(a.L[l], &dA, &dG, nullptr, nullptr);
        TraceJob T{};
        T.A = dry ? nullptr : a.A_ema[l];
        T.G = dry ? nullptr : a.G_ema[l];
        T.dA = dA; T.dG = dG;
        T.idx = l;
        tjobs.push_back(T);
        // dry runs only need distinct, well-aligned stand-in addresses for planning
        mats.push_back({T.A, dry ? (float *)nullptr : a.A_inv[l], dA, 3 * l + 1, 2 * l, a.L[l].bias != 0});
        mats.push_back({T.G, dry ? (float *)nullptr : a.G_inv[l], dG, 3 * l + 2, 2 * l + 1, false});
    }
    {
        Launch T{};
        T.kind = L_TRACE;
        T.off_a = plan.tab.add(tjobs.data(), tjobs.size() * sizeof(TraceJob));
        T.n = (int)tjobs.size();
        T.f0 = a.gamma;
        T.p0 = damp;
        T.p1 = a.pi_out;
        plan.launches.push_back(T);
    }
    plan_invert_mats(plan, arena, tun, mats, damp, a.info);
    plan.set_stream(first_launch, stream);
}

double chain_load(const kfac_layer &L)
{
    int dA, dG;
    layer_ok(L, &dA, &dG, nullptr, nullptr);
    auto cube = [](int n) { return n > kLeafMax ? (double)n * n * n : 0.0; };
    return cube(dA) + cube(dG);
}

// Deals layers (largest chains first) into n_groups groups of similar total n^3.
std::vector<std::vector<int>> deal_layers(const kfac_layer *L, std::vector<int> ids, int n_groups, int first_group)
{
    std::vector<std::vector<int>> groups(n_groups);
    std::stable_sort(ids.begin(), ids.end(), [&](int x, int y) { return chain_load(L[x]) > chain_load(L[y]); });
    std::vector<double> load(n_groups, 0.0);
    for (int l : ids) {
        int g = first_group;
        if (chain_load(L[l]) > 0.0)
            for (int q = first_group; q < n_groups; ++q)
                if (load[q] < load[g]) g = q;
        groups[g].push_back(l);
        load[g] += chain_load(L[l]);
    }
    return groups;
}

// Deals layers into two groups by the length of their chains instead: the number of dependent launches of a
// recursion grows with the size of the matrix (16 leaf inversions and 60 products for 4608, half of that for
// 2304, ...), and a levelled schedule is as long as its longest chain.  The matrices with more than half as
// many leaves as the largest one share the first group and advance together in launches of their own; all the
// others run level by level beside them on a second stream and are out of the way early.  (Measured,
// configuration 4: 5.8 ms against 6.1-6.2 ms for four groups of equal n^3 and for one group per size class:
// every further stream of small launches slows the long chains more than it hides.)
std::vector<std::vector<int>> deal_by_depth(const kfac_layer *L, std::vector<int> ids, int n_groups, int first_group)
{
    std::vector<std::vector<int>> groups(n_groups);
    auto leaves = [&](int l) {
        int dA, dG;
        layer_ok(L[l], &dA, &dG, nullptr, nullptr);
        return (std::max(dA - (L[l].bias ? 1 : 0), dG) + kLeafMax - 1) / kLeafMax;
    };
    int deepest = 1;
    for (int l : ids) deepest = std::max(deepest, leaves(l));
    const bool two = n_groups - first_group >= 2 && deepest > 2;
    for (int l : ids) groups[first_group + ((two && 2 * leaves(l) <= deepest) ? 1 : 0)].push_back(l);
    return groups;
}

// The recursion of one matrix is a long dependent chain of small launches.  Layers are dealt
// into up to inv_streams groups; each group has its own levelled schedule on its own stream,
// so the serial parts of one chain overlap the large products of another.  Group 0 runs on the
// context's stream; the others start after everything enqueued before (sync event 0) and are
// joined at the end (events 1..3).  Scratch of different groups never overlaps.
void plan_invert(Plan &plan, Arena &arena, const Tunables &tun, const InvertArgs &a, bool dry)
{
    float *damp = (float *)arena.take((size_t)3 * a.n_layers * sizeof(float));
    if (a.info || dry) {
        Launch Z{};
        Z.kind = L_ZERO;
        Z.p0 = a.info;
        Z.n = 2 * a.n_layers;
        plan.launches.push_back(Z);
    }
    const int n_groups = std::max(1, std::min(tun.inv_streams, 4));
    std::vector<int> all(a.n_layers);
    for (int l = 0; l < a.n_layers; ++l) all[l] = l;
    std::vector<std::vector<int>> groups = tun.by_depth ? deal_by_depth(a.L, all, n_groups, 0) : deal_layers(a.L, all, n_groups, 0);
    bool forked = false;
    // auxiliary groups first, so that their launches are enqueued before the main chain's
    for (int gi = 0; gi < n_groups; ++gi) {
        const int g = (gi + 1) % n_groups;
        if (groups[g].empty()) continue;
        if (g > 0) {
            if (!forked) plan.sync(L_RECORD, 0, 0);
            forked = true;
            plan.sync(L_WAIT, 0, g);
        }
        arena.used = align_up(arena.peak, kAlign);
        plan_invert_group(plan, arena, tun, a, dry, groups[g], damp, g);
        if (g > 0) plan.sync(L_RECORD, g, g);
    }
    for (int g = 1; g < n_groups; ++g)
        if (!groups[g].empty()) plan.sync(L_WAIT, g, 0);
}

// ---------------------------------------------------------------- preconditioning planner
struct PrecondArgs {
    int n_layers;
    const kfac_layer *L;
    const float *const *G_inv;
    const float *const *A_inv;
    const float *const *grad_W;
    float *const *out;
};

// `subset` (or null for all): the layers of `a` to precondition.
void plan_precondition(Plan &plan, Arena &arena, const Tunables &tun, const PrecondArgs &a, bool dry,
                       const std::vector<int> *subset = nullptr)
{
    // phase 1: Vt = A_inv * grad_W^T  ([dA, dG]);  phase 2: out = G_inv * Vt^T  ([dG, dA])
    std::vector<GemmProblem> p1, p2;
    const int n_sel = subset ? (int)subset->size() : a.n_layers;
    for (int q = 0; q < n_sel; ++q) {
        const int l = subset ? (*subset)[q] : q;
        int dA, dG;
        layer_ok(a.L[l], &dA, &dG, nullptr, nullptr);
        const long long ldv = align_up((size_t)dG, 4);
        float *Vt = (float *)arena.take((size_t)dA * ldv * sizeof(float));
        GemmProblem P{};
        P.a = plain_operand(dry ? nullptr : a.A_inv[l], dA, dA, dA);
        P.b = plain_operand(dry ? nullptr : a.grad_W[l], dA, dG, dA);
        P.C = Vt; P.ldc = ldv; P.Ct = nullptr;
        P.M = dA; P.N = dG; P.K = dA; P.flags = 0;
        P.alpha = 1.f; P.beta = 0.f;
        P.tile_cfg = choose_tile_cfg(P.M, P.N, P.K, (P.flags & GEMM_SYM) != 0);
        finish_problem(P);
        p1.push_back(P);
        GemmProblem Q{};
        Q.a = plain_operand(dry ? nullptr : a.G_inv[l], dG, dG, dG);
        Q.b = plain_operand(Vt, ldv, dA, dG);
        Q.C = dry ? nullptr : a.out[l]; Q.ldc = dA; Q.Ct = nullptr;
        Q.M = dG; Q.N = dA; Q.K = dG; Q.flags = 0;
        Q.alpha = 1.f; Q.beta = 0.f;
        Q.tile_cfg = choose_tile_cfg(Q.M, Q.N, Q.K, false);
        finish_problem(Q);
        p2.push_back(Q);
    }
    emit_gemm_phase(plan, arena, tun, p1, 0, true, true);
    emit_gemm_phase(plan, arena, tun, p2, 0, true, true);
}

// ---------------------------------------------------------------- fused step planner
// One K-FAC step as a single dependency graph: factors of every layer, inverses of the
// layers selected by `mask` (null: all), preconditioned gradients of every layer.  The
// results are those of the three separate calls; the difference is the schedule.  The
// inversion of a large factor is a long chain of mostly small launches that leaves the GPU
// idle, while the factor contractions are throughput bound.  So the layers are built in
// classes, longest chains first:
//   class 0: a factor of at least 2 * early_n   (event 4)
//   class 1: a factor of at least early_n       (event 5)
//   rest
// all on the context's stream, and the chains of a class start on auxiliary streams as soon
// as its factors exist.  (A grid of thousands of matrix-kernel workgroups leaves no compute
// unit with room for another workgroup, so the chains mostly advance between the big
// launches, not underneath them; what this order buys is that the longest chains are not also
// the last to start.)  The rest is inverted on the context's stream.
void plan_step(Plan &plan, Arena &arena, const Tunables &tun, const StatsArgs &st, const InvertArgs &inv,
               const uint8_t *mask, const PrecondArgs &pc, bool dry)
{
    const int n = st.n_layers;
    float *damp = (float *)arena.take((size_t)3 * n * sizeof(float));
    if (inv.info || dry) {
        Launch Z{};
        Z.kind = L_ZERO;
        Z.p0 = inv.info;
        Z.n = 2 * n;
        plan.launches.push_back(Z);
    }
    const int n_aux = std::max(0, std::min(tun.inv_streams, 4) - 1);
    std::vector<int> cls[2], late, late_inv;
    for (int l = 0; l < n; ++l) {
        int dA, dG;
        layer_ok(st.L[l], &dA, &dG, nullptr, nullptr);
        const bool inverted = !mask || mask[l];
        const int big = std::max(dA, dG);
        if (inverted && n_aux > 0 && big >= tun.early_n) cls[big >= 2 * tun.early_n ? 0 : 1].push_back(l);
        else {
            late.push_back(l);
            if (inverted) late_inv.push_back(l);
        }
    }
    if (cls[0].empty()) std::swap(cls[0], cls[1]);
    // auxiliary streams per class: with two classes the first (few, longest chains) gets one
    int aux_of[2][2] = {{1, n_aux}, {0, -1}};   // [class][first, last]
    if (!cls[1].empty()) {
        if (n_aux >= 2) { aux_of[0][1] = 1; aux_of[1][0] = 2; aux_of[1][1] = n_aux; }
        else { cls[0].insert(cls[0].end(), cls[1].begin(), cls[1].end()); cls[1].clear(); }
    }
    const size_t mark0 = arena.used;
    // Factor phases in class order.  With auxiliary streams the phases are pipelined: the
    // operand rewrites of the next phase run (on the last auxiliary stream, idle until its chain
    // starts) under the matrix launches of the current one, and what follows the matrix launches
    // of a class runs at the head of the first stream of its chains, under the matrix launches
    // of the next phase.  Each phase then needs scratch of its own.
    //   event 6: the call's tables are on the device (recorded first on the context's stream)
    //   events 7, 8: rewrites of the second / third phase done
    //   events 9 + c: matrix launches of class c done;  events 4 + c: factors of class c complete
    const std::vector<int> *phases[3] = {&cls[0], &cls[1], &late};
    const bool pipe = n_aux > 0 && tun.pipe;
    if (pipe) plan.sync(L_RECORD, 6, 0);
    // Beside running chains, the matrix launches of the later phases are cut into successive parts
    // of about chunk_gf GFLOP (at most 8): a chain's workgroups mostly get compute units where a
    // large launch drains, so more such points let the chains advance (configuration 4: -2 % on
    // the step, although the parts cost the factor contractions themselves 5-10 %).  Only when
    // the early chains are long against the contractions they run beside (n^3 per inverse against
    // K d^2 per factor); with few or short chains the parts only cost (configuration 5: +2.7 %).
    auto factor_gf = [&](int l) {
        int dA, dG, h, w;
        layer_ok(st.L[l], &dA, &dG, &h, &w);
        return 1e-9 * (double)st.L[l].N * h * w * ((double)dA * dA + (double)dG * dG);
    };
    bool chunked = false;
    if (tun.chunk_gf > 0) {
        double inv_early = 0, gf_later = 0;
        for (int c = 0; c < 2; ++c)
            for (int l : cls[c]) {
                int dA, dG;
                layer_ok(st.L[l], &dA, &dG, nullptr, nullptr);
                inv_early += 1e-9 * ((double)dA * dA * dA + (double)dG * dG * dG);
            }
        for (int l : cls[1]) gf_later += factor_gf(l);
        for (int l : late) gf_later += factor_gf(l);
        chunked = gf_later <= 2.0 * inv_early;
    }
    bool pre_waited = false;
    int n_phase = 0;
    for (int ph = 0; ph < 3; ++ph) {
        if (phases[ph]->empty()) continue;
        StatsSplit sp{0, 0, 0, 0, 1};
        if (pipe && n_phase > 0 && chunked) {
            double gf = 0;
            for (int l : *phases[ph]) gf += factor_gf(l);
            sp.gemm_chunks = std::min(8, std::max(1, (int)std::lround(gf / tun.chunk_gf)));
        }
        if (pipe) {
            if (n_phase > 0) {
                sp.pre_stream = n_aux;
                sp.ev_pre = 6 + n_phase;
                if (!pre_waited) plan.sync(L_WAIT, 6, n_aux);
                pre_waited = true;
            }
            if (ph < 2) { sp.post_stream = aux_of[ph][0]; sp.ev_gemm = 9 + ph; }
        } else {
            arena.release_to(mark0);   // one stream: each phase starts after the previous one has finished
        }
        plan_stats(plan, arena, tun, st, dry, phases[ph], &sp);
        if (ph < 2) plan.sync(L_RECORD, 4 + ph, pipe ? aux_of[ph][0] : 0);
        ++n_phase;
    }
    bool joined[4] = {false, false, false, false};
    const int early_classes = (cls[0].empty() ? 0 : 1) + (cls[1].empty() ? 0 : 1);
    for (int c = 0; c < 2; ++c) {
        if (cls[c].empty()) continue;
        const int g0 = aux_of[c][0], g1 = aux_of[c][1];
        std::vector<std::vector<int>> groups = deal_layers(st.L, cls[c], g1 + 1, g0);
        for (int g = g0; g <= g1; ++g) {
            if (groups[g].empty() && g != g0) continue;
            if (g != g0 || !pipe) plan.sync(L_WAIT, 4 + c, g);   // (pipelined: the first stream of the class completed the factors itself)
            arena.used = align_up(arena.peak, kAlign);   // concurrent with everything else: own scratch
            plan_invert_group(plan, arena, tun, inv, dry, groups[g], damp, g);
            plan.sync(L_RECORD, g, g);
            joined[g] = true;
        }
    }
    arena.used = align_up(arena.peak, kAlign);
    if (early_classes == 0 && n_aux > 0 && late_inv.size() > 1) {
        // no layer large enough for a class of its own (or none of them inverted): the inversions start when all
        // factors exist, the longest chains on the first auxiliary stream and the others here (as kfac_invert)
        std::vector<std::vector<int>> groups = deal_by_depth(st.L, late_inv, 2, 0);
        if (!groups[0].empty() && !groups[1].empty()) {
            plan.sync(L_RECORD, 4, 0);
            plan.sync(L_WAIT, 4, 1);
            plan_invert_group(plan, arena, tun, inv, dry, groups[0], damp, 1);
            plan.sync(L_RECORD, 1, 1);
            arena.used = align_up(arena.peak, kAlign);
            plan_invert_group(plan, arena, tun, inv, dry, groups[1], damp, 0);
            plan.sync(L_WAIT, 1, 0);
        } else {
            plan_invert_group(plan, arena, tun, inv, dry, late_inv, damp, 0);
        }
    } else {
        plan_invert_group(plan, arena, tun, inv, dry, late_inv, damp, 0);
    }
    // Preconditioning in the order in which the inverses arrive: the layers inverted on this
    // stream first, then each class once its chains have been joined, so that these products
    // fill the time in which only the longest chain is still running.  (Scratch beyond
    // everything handed out so far: chains on other streams are still using theirs.)
    if (early_classes == 0) arena.release_to(mark0);   // nothing else is running: reuse the scratch
    else arena.used = align_up(arena.peak, kAlign);
    if (!late.empty()) plan_precondition(plan, arena, tun, pc, dry, &late);
    for (int c = 1; c >= 0; --c) {
        if (cls[c].empty()) continue;
        for (int g = aux_of[c][0]; g <= aux_of[c][1]; ++g)
            if (joined[g]) plan.sync(L_WAIT, g, 0);
        plan_precondition(plan, arena, tun, pc, dry, &cls[c]);
    }
}

// ---------------------------------------------------------------- execution
constexpr size_t kPinnedSlotBytes = (size_t)1 << 20;   // table space per staging slot allocated up front

// Internal streams, the events that order them, and the pinned staging ring with its events.
// Called from kfac_create when a device is present, so that no call allocates anything later
// (except a call whose tables outgrow a staging slot); otherwise from the first call that launches.
kfac_status prepare_resources(kfac_ctx *ctx)
{
    if (ctx->resources_ready) return KFAC_OK;
    for (int q = 0; q < 3; ++q)
        if (!ctx->aux[q] && hipStreamCreateWithFlags(&ctx->aux[q], hipStreamNonBlocking) != hipSuccess) return KFAC_ERR_DEVICE;
    for (int q = 0; q < kSyncEvents; ++q)
        if (!ctx->sync_ev[q] && hipEventCreateWithFlags(&ctx->sync_ev[q], hipEventDisableTiming) != hipSuccess)
            return KFAC_ERR_DEVICE;
    for (int slot = 0; slot < ctx->tun.slots; ++slot) {
        if (!ctx->ev[slot] && hipEventCreateWithFlags(&ctx->ev[slot], hipEventDisableTiming) != hipSuccess)
            return KFAC_ERR_DEVICE;
        if (!ctx->pinned[slot]) {
            void *p = nullptr;
            if (hipHostMalloc(&p, kPinnedSlotBytes, hipHostMallocDefault) != hipSuccess) return KFAC_ERR_DEVICE;
            ctx->pinned[slot] = (char *)p;
            ctx->pinned_bytes[slot] = kPinnedSlotBytes;
        }
    }
    ctx->resources_ready = true;
    return KFAC_OK;
}

// The staging slot of this call: waits until the device has consumed what the slot held (the call
// `slots` calls back), and grows the slot if this call's tables do not fit.
kfac_status ensure_slot(kfac_ctx *ctx, int slot, size_t bytes)
{
    if (ctx->ev_used[slot] && hipEventSynchronize(ctx->ev[slot]) != hipSuccess) return KFAC_ERR_DEVICE;
    if (ctx->pinned_bytes[slot] < bytes) {
        if (ctx->pinned[slot]) (void)hipHostFree(ctx->pinned[slot]);
        ctx->pinned[slot] = nullptr;
        ctx->pinned_bytes[slot] = 0;
        void *p = nullptr;
        if (hipHostMalloc(&p, bytes, hipHostMallocDefault) != hipSuccess) return KFAC_ERR_DEVICE;
        ctx->pinned[slot] = (char *)p;
        ctx->pinned_bytes[slot] = bytes;
    }
    return KFAC_OK;
}

kfac_status run_plan(kfac_ctx *ctx, Plan &plan, Arena &arena)
{
    // tables go behind the scratch slices
    const size_t tab_bytes = plan.tab.buf.size();
    char *tab_dev = (char *)arena.take_tail(tab_bytes + 16);
    if (arena.peak > ctx->ws_bytes) return KFAC_ERR_WORKSPACE;
    hipStream_t s = ctx->stream;
    {
        kfac_status st = prepare_resources(ctx);
        if (st != KFAC_OK) return st;
    }
    if (tab_bytes) {
        const int slot = ctx->next_slot;
        ctx->next_slot = (ctx->next_slot + 1) % ctx->tun.slots;
        kfac_status st = ensure_slot(ctx, slot, tab_bytes);
        if (st != KFAC_OK) return st;
        memcpy(ctx->pinned[slot], plan.tab.buf.data(), tab_bytes);
        if (hipMemcpyAsync(tab_dev, ctx->pinned[slot], tab_bytes, hipMemcpyHostToDevice, s) != hipSuccess)
            return KFAC_ERR_DEVICE;
        if (hipEventRecord(ctx->ev[slot], s) != hipSuccess) return KFAC_ERR_DEVICE;
        ctx->ev_used[slot] = true;
    }
    for (auto &L : plan.launches) {
        hipError_t e = hipSuccess;
        hipStream_t ls = s;
        if (L.stream > 0) ls = ctx->aux[L.stream - 1];
        if (L.kind == L_RECORD) {
            if (hipEventRecord(ctx->sync_ev[L.n], ls) != hipSuccess) return KFAC_ERR_DEVICE;
            continue;
        }
        if (L.kind == L_WAIT) {
            if (hipStreamWaitEvent(ls, ctx->sync_ev[L.n], 0) != hipSuccess) return KFAC_ERR_DEVICE;
            continue;
        }
        const bool timed = ctx->profiling && L.kind != L_ZERO;
        if (timed) {
            const size_t idx = ctx->prof.size();
            while (ctx->ev_pool.size() < 2 * (idx + 1)) {
                hipEvent_t ev;
                if (hipEventCreate(&ev) != hipSuccess) return KFAC_ERR_DEVICE;
                ctx->ev_pool.push_back(ev);
            }
            kfac_profile_entry pe{};
            switch (L.kind) {
                case L_GEMM: pe.kernel = L.dtype == 0 ? KFAC_K_GEMM_F32 : (L.dtype == 2 || L.dtype == 3) ? KFAC_K_GEMM_F32_SPLIT : KFAC_K_GEMM_BF16; break;
                case L_REDUCE: pe.kernel = KFAC_K_GEMM_REDUCE; break;
                case L_PATCH: pe.kernel = KFAC_K_PATCH; break;
                case L_TRACE: pe.kernel = KFAC_K_TRACE; break;
                case L_COPY: pe.kernel = KFAC_K_COPY_DAMP; break;
                case L_LEAF: pe.kernel = KFAC_K_LEAF_INVERSE; break;
                case L_ZERO: pe.kernel = KFAC_K_ZERO; break;
                case L_BN: pe.kernel = KFAC_K_BN_UNIT; break;
                case L_BNRED: pe.kernel = KFAC_K_BN_REDUCE; break;
                case L_PAD: pe.kernel = KFAC_K_PAD; break;
                case L_ASSEMBLE: pe.kernel = KFAC_K_ASSEMBLE; break;
                case L_BORDER: pe.kernel = KFAC_K_BORDER; break;
                case L_STALE: pe.kernel = KFAC_K_STALENESS; break;
                case L_PACK: pe.kernel = KFAC_K_PACK; break;
                case L_UPDATE: pe.kernel = KFAC_K_UPDATE; break;
                case L_BNFULL: pe.kernel = KFAC_K_BN_FULL; break;
                case L_LAYOUT: pe.kernel = KFAC_K_LAYOUT; break;
                case L_RECORD: case L_WAIT: break;
            }
            pe.variant = (L.kind == L_GEMM || L.kind == L_LEAF || L.kind == L_BNFULL) ? L.cfg : 0;
            pe.workgroups = (L.kind == L_TRACE || L.kind == L_LEAF) ? L.n : L.total_wgs;
            pe.flops = L.flops;
            pe.bytes = L.bytes;
            pe.stream = L.stream;
            ctx->prof.push_back(pe);
            if (hipEventRecord(ctx->ev_pool[2 * idx], ls) != hipSuccess) return KFAC_ERR_DEVICE;
        }
        switch (L.kind) {
            case L_GEMM:
                e = launch_gemm((const GemmProblem *)(tab_dev + L.off_a), (const int *)(tab_dev + L.off_b), L.n,
                                L.total_wgs, L.cfg, L.dtype, ls);
                break;
            case L_REDUCE:
                e = launch_gemm_reduce((const GemmProblem *)(tab_dev + L.off_a), (const int *)(tab_dev + L.off_b),
                                       L.n, L.total_wgs, ls);
                break;
            case L_PATCH:
                e = launch_patch((const PatchJob *)(tab_dev + L.off_a), L.n, L.total_wgs, ls);
                break;
            case L_PAD:
                e = L.cfg == 1 ? launch_pad_bf16((const PadJobBF16 *)(tab_dev + L.off_a), L.n, L.total_wgs, ls)
                               : launch_pad((const PadJob *)(tab_dev + L.off_a), L.n, L.total_wgs, ls);
                break;
            case L_ASSEMBLE:
                e = launch_assemble((const AssembleJob *)(tab_dev + L.off_a), L.n, L.total_wgs, ls);
                break;
            case L_BORDER:
                e = launch_border((const BorderJob *)(tab_dev + L.off_a), L.n, L.total_wgs, L.cfg, (const float *)L.p0,
                                  (int32_t *)L.p1, ls);
                break;
            case L_TRACE:
                e = launch_trace((const TraceJob *)(tab_dev + L.off_a), L.n, L.f0, (float *)L.p0, (float *)L.p1, ls);
                break;
            case L_COPY:
                e = launch_copy_damp((const CopyJob *)(tab_dev + L.off_a), L.n, L.total_wgs, (const float *)L.p0, ls);
                break;
            case L_LEAF:
                e = launch_leaf((const LeafJob *)(tab_dev + L.off_a), L.n, L.cfg, (const float *)L.p0,
                                (int32_t *)L.p1, ls);
                break;
            case L_ZERO:
                e = launch_zero_i32((int32_t *)L.p0, L.n, ls);
                break;
            case L_BN:
                e = launch_bn((const BnJob *)(tab_dev + L.off_a), L.n, L.total_wgs, L.cfg, L.f0, L.f1, ls);
                break;
            case L_BNRED:
                e = launch_bn_reduce((const BnReduceJob *)(tab_dev + L.off_a), L.n, L.total_wgs, L.cfg, L.dtype, ls);
                break;
            case L_LAYOUT:
                e = launch_nhwc_to_nchw((const LayoutJob *)(tab_dev + L.off_a), L.n, L.total_wgs, L.cfg, ls);
                break;
            case L_BNFULL:
                e = launch_bn_full((const BnFullJob *)(tab_dev + L.off_a), L.n, L.total_wgs, L.cfg, L.dtype, L.f0, L.f1,
                                   (float *)L.p0, ls);
                break;
            case L_UPDATE:
                e = launch_update((const UpdateJob *)(tab_dev + L.off_a), L.n, L.total_wgs, L.cfg, L.f0, L.f1, L.f0, ls);
                break;
            case L_PACK:
                e = launch_pack((const PackJob *)(tab_dev + L.off_a), L.n, L.total_wgs, L.dtype, L.cfg, L.p0, ls);
                break;
            case L_STALE:
                e = launch_staleness((const StaleJob *)(tab_dev + L.off_a), L.n, L.total_wgs, L.cfg, ls);
                break;
            case L_RECORD: case L_WAIT: break;
        }
        if (e != hipSuccess) return KFAC_ERR_DEVICE;
        if (timed && hipEventRecord(ctx->ev_pool[2 * ctx->prof.size() - 1], ls) != hipSuccess)
            return KFAC_ERR_DEVICE;
    }
    return KFAC_OK;
}

bool layers_ok(const kfac_layer *L, int n)
{
    if (!L || n < 1 || n > 65536) return false;
    for (int i = 0; i < n; ++i)
        if (!layer_ok(L[i], nullptr, nullptr, nullptr, nullptr)) return false;
    return true;
}

}  // namespace

// ------------------------------------------------------------------ C ABI
extern "C" {

const char *kfac_status_string(kfac_status s)
{
    switch (s) {
        case KFAC_OK: return "ok";
        case KFAC_ERR_INVALID: return "invalid argument";
        case KFAC_ERR_WORKSPACE: return "workspace too small";
        case KFAC_ERR_NOT_PD: return "matrix not positive definite";
        case KFAC_ERR_DEVICE: return "HIP runtime error";
    }
    return "unknown status";
}

kfac_status kfac_layer_dims(const kfac_layer *L, int32_t *dA, int32_t *dG, int32_t *h, int32_t *w)
{
    if (!L) return KFAC_ERR_INVALID;
    int a, g, hh, ww;
    if (!layer_ok(*L, &a, &g, &hh, &ww)) return KFAC_ERR_INVALID;
    if (dA) *dA = a;
    if (dG) *dG = g;
    if (h) *h = hh;
    if (w) *w = ww;
    return KFAC_OK;
}

size_t kfac_step_workspace_bytes(const kfac_layer *L, int32_t n_layers, kfac_dtype in, const uint8_t *invert_mask,
                                 const kfac_options *opt)
{
    if (!layers_ok(L, n_layers) || (in != KFAC_F32 && in != KFAC_BF16) || !options_ok(opt)) return 0;
    const Tunables tun(opt ? *opt : default_options());
    Plan plan; Arena arena(nullptr);
    StatsArgs st{n_layers, L, in, nullptr, nullptr, 0.5f, 0, nullptr, nullptr};
    InvertArgs iv{n_layers, L, nullptr, nullptr, 1e-3f, nullptr, nullptr, nullptr, nullptr};
    PrecondArgs pc{n_layers, L, nullptr, nullptr, nullptr, nullptr};
    plan_step(plan, arena, tun, st, iv, invert_mask, pc, true);
    arena.take_tail(plan.tab.buf.size() + 16);
    return arena.peak;
}

void kfac_options_default(kfac_options *opt)
{
    if (opt) *opt = default_options();
}

size_t kfac_workspace_bytes(const kfac_layer *L, int32_t n_layers, kfac_dtype in)
{
    return kfac_workspace_bytes_opt(L, n_layers, in, nullptr);
}

size_t kfac_workspace_bytes_opt(const kfac_layer *L, int32_t n_layers, kfac_dtype in, const kfac_options *opt)
{
    if (!layers_ok(L, n_layers) || (in != KFAC_F32 && in != KFAC_BF16) || !options_ok(opt)) return 0;
    Tunables tun(opt ? *opt : default_options());
    tun.worst_case_splits = true;
    size_t best = 0, sum_peaks = 0;
    {
        size_t stats_peak = 0;
        for (int nhwc = 0; nhwc < 2; ++nhwc) {   // NHWC inputs add the scratch of the tensors that are converted
            Plan plan; Arena arena(nullptr);
            StatsArgs a{n_layers, L, in, nullptr, nullptr, 0.5f, 0, nullptr, nullptr};
            a.nhwc = nhwc;
            plan_stats(plan, arena, tun, a, true);
            arena.take_tail(plan.tab.buf.size() + 16);
            stats_peak = std::max(stats_peak, arena.peak);
        }
        best = std::max(best, stats_peak);
        sum_peaks += stats_peak;
    }
    {
        Plan plan; Arena arena(nullptr);
        InvertArgs a{n_layers, L, nullptr, nullptr, 1e-3f, nullptr, nullptr, nullptr, nullptr};
        plan_invert(plan, arena, tun, a, true);
        arena.take_tail(plan.tab.buf.size() + 16);
        best = std::max(best, arena.peak);
        sum_peaks += arena.peak;
    }
    {
        Plan plan; Arena arena(nullptr);
        PrecondArgs a{n_layers, L, nullptr, nullptr, nullptr, nullptr};
        plan_precondition(plan, arena, tun, a, true);
        arena.take_tail(plan.tab.buf.size() + 16);
        best = std::max(best, arena.peak);
    }
    {
        // fused step, all layers inverted.  A partial mask moves layers between the factor phases
        // and the inversion groups, which changes tile choices and split-K scratch by a few percent
        // (searching over masks found 10 % above the full mask's plan at most): the sum of the
        // separate peaks plus a quarter covers that with room; kfac_step_workspace_bytes gives the
        // exact figure for one mask, and every call checks its own plan before it launches anything
        for (int nhwc = 0; nhwc < 2; ++nhwc) {
            Plan plan; Arena arena(nullptr);
            StatsArgs st{n_layers, L, in, nullptr, nullptr, 0.5f, 0, nullptr, nullptr};
            st.nhwc = nhwc;
            InvertArgs iv{n_layers, L, nullptr, nullptr, 1e-3f, nullptr, nullptr, nullptr, nullptr};
            PrecondArgs pc{n_layers, L, nullptr, nullptr, nullptr, nullptr};
            plan_step(plan, arena, tun, st, iv, nullptr, pc, true);
            arena.take_tail(plan.tab.buf.size() + 16);
            best = std::max(best, std::max(arena.peak, sum_peaks + sum_peaks / 4));
        }
    }
    // im2col of a single layer and the BatchNorm calls need table space only
    best = std::max(best, (size_t)1 << 20);
    return align_up(best + 4096, kAlign);
}

kfac_status kfac_create(kfac_ctx **out, void *hip_stream, void *workspace_dev, size_t workspace_bytes)
{
    return kfac_create_opt(out, hip_stream, workspace_dev, workspace_bytes, nullptr);
}

kfac_status kfac_create_opt(kfac_ctx **out, void *hip_stream, void *workspace_dev, size_t workspace_bytes,
                            const kfac_options *opt)
{
    if (!out) return KFAC_ERR_INVALID;
    *out = nullptr;
    if (!workspace_dev || workspace_bytes == 0 || ((uintptr_t)workspace_dev % kAlign) != 0) return KFAC_ERR_INVALID;
    if (!options_ok(opt)) return KFAC_ERR_INVALID;
    kfac_ctx *c = new (std::nothrow) kfac_ctx();
    if (!c) return KFAC_ERR_DEVICE;
    c->stream = (hipStream_t)hip_stream;
    c->ws = (char *)workspace_dev;
    c->ws_bytes = workspace_bytes;
    c->tun = Tunables(opt ? *opt : default_options());
    for (int i = 0; i < kSlots; ++i) {
        c->pinned[i] = nullptr;
        c->pinned_bytes[i] = 0;
        c->ev[i] = nullptr;
        c->ev_used[i] = false;
    }
    for (int q = 0; q < 3; ++q) c->aux[q] = nullptr;
    for (int q = 0; q < kSyncEvents; ++q) c->sync_ev[q] = nullptr;
    c->next_slot = 0;
    c->profiling = false;
    c->resources_ready = false;
    // streams, events and the staging ring now, if there is a device to create them on (a machine
    // without one still gets a context: argument validation needs no GPU)
    int n_dev = 0;
    if (hipGetDeviceCount(&n_dev) == hipSuccess && n_dev > 0) {
        if (prepare_resources(c) != KFAC_OK) {
            kfac_destroy(c);
            return KFAC_ERR_DEVICE;
        }
    } else {
        (void)hipGetLastError();   // (the failed device query is not this library's caller's error)
    }
    *out = c;
    return KFAC_OK;
}

void kfac_destroy(kfac_ctx *ctx)
{
    if (!ctx) return;
    for (int i = 0; i < kSlots; ++i) {
        if (ctx->ev[i]) {
            if (ctx->ev_used[i]) (void)hipEventSynchronize(ctx->ev[i]);
            (void)hipEventDestroy(ctx->ev[i]);
        }
        if (ctx->pinned[i]) (void)hipHostFree(ctx->pinned[i]);
    }
    for (auto ev : ctx->ev_pool) (void)hipEventDestroy(ev);
    for (int q = 0; q < 3; ++q)
        if (ctx->aux[q]) {
            (void)hipStreamSynchronize(ctx->aux[q]);
            (void)hipStreamDestroy(ctx->aux[q]);
        }
    for (int q = 0; q < kSyncEvents; ++q)
        if (ctx->sync_ev[q]) (void)hipEventDestroy(ctx->sync_ev[q]);
    delete ctx;
}

kfac_status kfac_profile_enable(kfac_ctx *ctx, int32_t on)
{
    if (!ctx) return KFAC_ERR_INVALID;
    ctx->profiling = on != 0;
    ctx->prof.clear();
    return KFAC_OK;
}

int32_t kfac_profile_read(kfac_ctx *ctx, kfac_profile_entry *out, int32_t max_entries)
{
    if (!ctx || (max_entries > 0 && !out) || max_entries < 0) return -1;
    const int32_t n = (int32_t)ctx->prof.size();
    if (n == 0) return 0;
    if (hipStreamSynchronize(ctx->stream) != hipSuccess) return -1;
    for (int32_t i = 0; i < n; ++i) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, ctx->ev_pool[2 * i], ctx->ev_pool[2 * i + 1]) != hipSuccess) return -1;
        ctx->prof[i].ms = ms;
        float t0 = 0.f;
        if (i > 0 && hipEventElapsedTime(&t0, ctx->ev_pool[0], ctx->ev_pool[2 * i]) != hipSuccess) return -1;
        ctx->prof[i].start_ms = t0;
        if (i < max_entries) out[i] = ctx->prof[i];
    }
    ctx->prof.clear();
    return n;
}

kfac_status kfac_im2col(kfac_ctx *ctx, const kfac_layer *L, kfac_dtype dt, const void *act, void *patches,
                        int64_t ld)
{
    if (!ctx || !L || !act || !patches) return KFAC_ERR_INVALID;
    if (dt != KFAC_F32 && dt != KFAC_BF16) return KFAC_ERR_INVALID;
    int dA, dG, h, w;
    if (!layer_ok(*L, &dA, &dG, &h, &w)) return KFAC_ERR_INVALID;
    const int hw = h * w;
    if (ld < (int64_t)L->N * hw) return KFAC_ERR_INVALID;
    Plan plan; Arena arena(ctx->ws);
    PatchJob J = make_patch_job(act, patches, ld, L->N, L->c_in, L->k, L->stride, L->pad, L->h_in, L->w_in, h, w,
                                dt == KFAC_BF16 ? 2 : 4);
    J.wg_start = 0;
    Launch Lc{};
    Lc.kind = L_PATCH;
    Lc.bytes = (double)J.esize * ((double)L->N * L->c_in * L->h_in * L->w_in + (double)L->c_in * L->k * L->k * L->N * hw);
    Lc.off_a = plan.tab.add(&J, sizeof(J));
    Lc.n = 1;
    Lc.total_wgs = patch_job_wgs(J);
    plan.launches.push_back(Lc);
    return run_plan(ctx, plan, arena);
}

static kfac_status stats_call(int nhwc, kfac_ctx *ctx, int32_t n_layers, const kfac_layer *L, kfac_dtype in,
                       const void *const *act, const void *const *grad_out, float decay, int32_t g_spatial_mean,
                       float *const *A_ema, float *const *G_ema)
{
    if (!ctx || !layers_ok(L, n_layers)) return KFAC_ERR_INVALID;
    if (in != KFAC_F32 && in != KFAC_BF16) return KFAC_ERR_INVALID;
    if (!(decay >= 0.0f && decay < 1.0f)) return KFAC_ERR_INVALID;
    if (!act && !grad_out) return KFAC_ERR_INVALID;
    for (int l = 0; l < n_layers; ++l) {
        if (act && act[l] && (!A_ema || !A_ema[l])) return KFAC_ERR_INVALID;
        if (grad_out && grad_out[l] && (!G_ema || !G_ema[l])) return KFAC_ERR_INVALID;
        const size_t es = in == KFAC_BF16 ? 2 : 4;
        if (act && act[l] && ((uintptr_t)act[l] % es) != 0) return KFAC_ERR_INVALID;
        if (grad_out && grad_out[l] && ((uintptr_t)grad_out[l] % es) != 0) return KFAC_ERR_INVALID;
    }
    Plan plan; Arena arena(ctx->ws);
    StatsArgs a{n_layers, L, in, act, grad_out, decay, g_spatial_mean != 0, A_ema, G_ema};
    a.nhwc = nhwc;
    plan_stats(plan, arena, ctx->tun, a, false);
    return run_plan(ctx, plan, arena);
}

kfac_status kfac_stats(kfac_ctx *ctx, int32_t n_layers, const kfac_layer *L, kfac_dtype in,
                       const void *const *act, const void *const *grad_out, float decay, int32_t g_spatial_mean,
                       float *const *A_ema, float *const *G_ema)
{
    return stats_call(0, ctx, n_layers, L, in, act, grad_out, decay, g_spatial_mean, A_ema, G_ema);
}

kfac_status kfac_stats_nhwc(kfac_ctx *ctx, int32_t n_layers, const kfac_layer *L, kfac_dtype in,
                            const void *const *act, const void *const *grad_out, float decay, int32_t g_spatial_mean,
                            float *const *A_ema, float *const *G_ema)
{
    return stats_call(1, ctx, n_layers, L, in, act, grad_out, decay, g_spatial_mean, A_ema, G_ema);
}

kfac_status kfac_invert(kfac_ctx *ctx, int32_t n_layers, const kfac_layer *L, const float *const *A_ema,
                        const float *const *G_ema, float gamma, float *const *A_inv, float *const *G_inv,
                        float *pi_out, int32_t *info)
{
    if (!ctx || !layers_ok(L, n_layers)) return KFAC_ERR_INVALID;
    if (!A_ema || !G_ema || !A_inv || !G_inv) return KFAC_ERR_INVALID;
    if (!(gamma >= 0.0f) || !std::isfinite(gamma)) return KFAC_ERR_INVALID;
    for (int l = 0; l < n_layers; ++l) {
        if (!A_ema[l] || !G_ema[l] || !A_inv[l] || !G_inv[l]) return KFAC_ERR_INVALID;
        if (A_ema[l] == A_inv[l] || G_ema[l] == G_inv[l]) return KFAC_ERR_INVALID;
    }
    Plan plan; Arena arena(ctx->ws);
    InvertArgs a{n_layers, L, A_ema, G_ema, gamma, A_inv, G_inv, pi_out, info};
    plan_invert(plan, arena, ctx->tun, a, false);
    return run_plan(ctx, plan, arena);
}

kfac_status kfac_precondition(kfac_ctx *ctx, int32_t n_layers, const kfac_layer *L, const float *const *G_inv,
                              const float *const *A_inv, const float *const *grad_W, float *const *out)
{
    if (!ctx || !layers_ok(L, n_layers)) return KFAC_ERR_INVALID;
    if (!G_inv || !A_inv || !grad_W || !out) return KFAC_ERR_INVALID;
    for (int l = 0; l < n_layers; ++l)
        if (!G_inv[l] || !A_inv[l] || !grad_W[l] || !out[l]) return KFAC_ERR_INVALID;
    Plan plan; Arena arena(ctx->ws);
    PrecondArgs a{n_layers, L, G_inv, A_inv, grad_W, out};
    plan_precondition(plan, arena, ctx->tun, a, false);
    return run_plan(ctx, plan, arena);
}

static kfac_status step_call(int nhwc, kfac_ctx *ctx, int32_t n_layers, const kfac_layer *L, kfac_dtype in,
                      const void *const *act, const void *const *grad_out, float decay, int32_t g_spatial_mean,
                      float *const *A_ema, float *const *G_ema, const uint8_t *invert_mask, float gamma,
                      float *const *A_inv, float *const *G_inv, float *pi_out, int32_t *info,
                      const float *const *grad_W, float *const *out)
{
    if (!ctx || !layers_ok(L, n_layers)) return KFAC_ERR_INVALID;
    if (in != KFAC_F32 && in != KFAC_BF16) return KFAC_ERR_INVALID;
    if (!(decay >= 0.0f && decay < 1.0f)) return KFAC_ERR_INVALID;
    if (!(gamma >= 0.0f) || !std::isfinite(gamma)) return KFAC_ERR_INVALID;
    if (!act || !grad_out || !A_ema || !G_ema || !A_inv || !G_inv || !grad_W || !out) return KFAC_ERR_INVALID;
    const size_t es = in == KFAC_BF16 ? 2 : 4;
    for (int l = 0; l < n_layers; ++l) {
        if (!act[l] || !grad_out[l] || !A_ema[l] || !G_ema[l] || !A_inv[l] || !G_inv[l] || !grad_W[l] || !out[l])
            return KFAC_ERR_INVALID;
        if (((uintptr_t)act[l] % es) != 0 || ((uintptr_t)grad_out[l] % es) != 0) return KFAC_ERR_INVALID;
        if (A_ema[l] == A_inv[l] || G_ema[l] == G_inv[l]) return KFAC_ERR_INVALID;
    }
    Plan plan; Arena arena(ctx->ws);
    StatsArgs st{n_layers, L, in, act, grad_out, decay, g_spatial_mean != 0, A_ema, G_ema};
    st.nhwc = nhwc;
    InvertArgs iv{n_layers, L, A_ema, G_ema, gamma, A_inv, G_inv, pi_out, info};
    PrecondArgs pc{n_layers, L, G_inv, A_inv, grad_W, out};
    plan_step(plan, arena, ctx->tun, st, iv, invert_mask, pc, false);
    return run_plan(ctx, plan, arena);
}

kfac_status kfac_step(kfac_ctx *ctx, int32_t n_layers, const kfac_layer *L, kfac_dtype in,
                      const void *const *act, const void *const *grad_out, float decay, int32_t g_spatial_mean,
                      float *const *A_ema, float *const *G_ema, const uint8_t *invert_mask, float gamma,
                      float *const *A_inv, float *const *G_inv, float *pi_out, int32_t *info,
                      const float *const *grad_W, float *const *out)
{
    return step_call(0, ctx, n_layers, L, in, act, grad_out, decay, g_spatial_mean, A_ema, G_ema, invert_mask, gamma,
                     A_inv, G_inv, pi_out, info, grad_W, out);
}

kfac_status kfac_step_nhwc(kfac_ctx *ctx, int32_t n_layers, const kfac_layer *L, kfac_dtype in,
                           const void *const *act, const void *const *grad_out, float decay, int32_t g_spatial_mean,
                           float *const *A_ema, float *const *G_ema, const uint8_t *invert_mask, float gamma,
                           float *const *A_inv, float *const *G_inv, float *pi_out, int32_t *info,
                           const float *const *grad_W, float *const *out)
{
    return step_call(1, ctx, n_layers, L, in, act, grad_out, decay, g_spatial_mean, A_ema, G_ema, invert_mask, gamma,
                     A_inv, G_inv, pi_out, info, grad_W, out);
}

kfac_status bn_unitwise_precondition(kfac_ctx *ctx, int32_t n_layers, int32_t N, const int32_t *C,
                                     const float *const *g_gamma, const float *const *g_beta, float decay,
                                     float lambda, float *const *F_ema, float *const *out_gamma,
                                     float *const *out_beta)
{
    if (!ctx || n_layers < 1 || n_layers > 65536 || N < 1 || !C) return KFAC_ERR_INVALID;
    if (!g_gamma || !g_beta || !F_ema || !out_gamma || !out_beta) return KFAC_ERR_INVALID;
    if (!(decay >= 0.0f && decay < 1.0f) || !(lambda >= 0.0f) || !std::isfinite(lambda)) return KFAC_ERR_INVALID;
    std::vector<BnJob> jobs;
    int wgs = 0;
    for (int l = 0; l < n_layers; ++l) {
        if (C[l] < 1 || C[l] > (1 << 24)) return KFAC_ERR_INVALID;
        if (!g_gamma[l] || !g_beta[l] || !F_ema[l] || !out_gamma[l] || !out_beta[l]) return KFAC_ERR_INVALID;
        BnJob J{};
        J.g_gamma = g_gamma[l]; J.g_beta = g_beta[l];
        J.F_ema = F_ema[l]; J.out_gamma = out_gamma[l]; J.out_beta = out_beta[l];
        J.C = C[l];
        J.wg_start = wgs;
        wgs += (C[l] + 255) / 256;
        jobs.push_back(J);
    }
    Plan plan; Arena arena(ctx->ws);
    Launch Lc{};
    Lc.kind = L_BN;
    for (auto &J : jobs) Lc.bytes += 8.0 * N * J.C + 32.0 * J.C;
    Lc.off_a = plan.tab.add(jobs.data(), jobs.size() * sizeof(BnJob));
    Lc.n = n_layers;
    Lc.total_wgs = wgs;
    Lc.cfg = N;
    Lc.f0 = decay;
    Lc.f1 = lambda;
    plan.launches.push_back(Lc);
    return run_plan(ctx, plan, arena);
}

namespace {
struct BnFullArgs {
    int n_layers, N;
    const int32_t *C;
    const float *const *g_gamma, *const *g_beta;
    float decay, lambda;
    float *const *F_ema;
    const uint8_t *invert_mask;
    float *const *F_inv;
    int32_t *info;
    float *const *out_gamma, *const *out_beta;
};

// factor update -> mean gradient and damping -> inversions (dealt by n^3 onto the context's
// stream and the auxiliary ones, as kfac_invert does) -> u = F_inv gbar
void plan_bn_full(Plan &plan, Arena &arena, const Tunables &tun, const BnFullArgs &a, bool dry)
{
    const int n = a.n_layers;
    float *damp = (float *)arena.take((size_t)n * sizeof(float));
    std::vector<BnFullJob> jobs(n);
    long long wgs[3] = {0, 0, 0};
    double bytes[3] = {0, 0, 0};
    std::vector<int> inv_ids;
    for (int l = 0; l < n; ++l) {
        BnFullJob &J = jobs[l];
        const long long d = 2LL * a.C[l];
        const bool inv = !a.invert_mask || a.invert_mask[l];
        J.g_gamma = dry ? nullptr : a.g_gamma[l];
        J.g_beta = dry ? nullptr : a.g_beta[l];
        J.F_ema = dry ? nullptr : a.F_ema[l];
        J.F_inv = dry ? nullptr : a.F_inv[l];
        J.out_gamma = dry ? nullptr : a.out_gamma[l];
        J.out_beta = dry ? nullptr : a.out_beta[l];
        J.gbar = (float *)arena.take((size_t)d * sizeof(float));
        J.C = a.C[l];
        J.damp_idx = inv ? l : -1;
        const long long tiles = (d + 63) / 64;
        const long long w[3] = {tiles * tiles, (d + 255) / 256, (d + 3) / 4};
        for (int q = 0; q < 3; ++q) { J.wg_start[q] = (int)wgs[q]; wgs[q] += w[q]; }
        bytes[0] += (a.decay == 0.f ? 4.0 : 8.0) * d * d + 4.0 * a.N * d * 2 * tiles;
        bytes[1] += 4.0 * a.N * d + 4.0 * d;
        bytes[2] += 4.0 * d * d + 8.0 * d;
        if (inv) inv_ids.push_back(l);
    }
    const size_t off = plan.tab.add(jobs.data(), jobs.size() * sizeof(BnFullJob));
    auto pass = [&](int q) {
        Launch Lc{};
        Lc.kind = L_BNFULL;
        Lc.off_a = off;
        Lc.n = n;
        Lc.total_wgs = (int)wgs[q];
        Lc.cfg = q;
        Lc.dtype = a.N;
        Lc.f0 = a.decay;
        Lc.f1 = a.lambda;
        Lc.p0 = damp;
        Lc.bytes = bytes[q];
        plan.launches.push_back(Lc);
    };
    pass(0);
    pass(1);
    if (a.info || dry) {
        Launch Z{};
        Z.kind = L_ZERO;
        Z.p0 = a.info;
        Z.n = n;
        plan.launches.push_back(Z);
    }
    if (!inv_ids.empty()) {
        const int n_groups = std::max(1, std::min(tun.inv_streams, 4));
        auto cube = [&](int l) { const double d = 2.0 * a.C[l]; return d > kLeafMax ? d * d * d : 0.0; };
        std::stable_sort(inv_ids.begin(), inv_ids.end(), [&](int x, int y) { return cube(x) > cube(y); });
        std::vector<std::vector<InvMatrix>> groups(n_groups);
        std::vector<double> load(n_groups, 0.0);
        for (int l : inv_ids) {
            int g = 0;
            if (cube(l) > 0.0)
                for (int q = 0; q < n_groups; ++q)
                    if (load[q] < load[g]) g = q;
            groups[g].push_back({jobs[l].F_ema, dry ? (float *)nullptr : a.F_inv[l], 2 * a.C[l], l, l, false});
            load[g] += cube(l);
        }
        bool forked = false;
        for (int gi = 0; gi < n_groups; ++gi) {
            const int g = (gi + 1) % n_groups;   // auxiliary chains are enqueued before the main one
            if (groups[g].empty()) continue;
            if (g > 0) {
                if (!forked) plan.sync(L_RECORD, 0, 0);
                forked = true;
                plan.sync(L_WAIT, 0, g);
            }
            arena.used = align_up(arena.peak, kAlign);   // scratch of concurrent chains stays apart
            const size_t first = plan.launches.size();
            plan_invert_mats(plan, arena, tun, groups[g], damp, a.info);
            plan.set_stream(first, g);
            if (g > 0) plan.sync(L_RECORD, g, g);
        }
        for (int g = 1; g < n_groups; ++g)
            if (!groups[g].empty()) plan.sync(L_WAIT, g, 0);
    }
    pass(2);
}

bool bn_full_dims_ok(int32_t n_layers, int32_t N, const int32_t *C)
{
    if (n_layers < 1 || n_layers > 65536 || N < 1 || N > (1 << 20) || !C) return false;
    long long tiles = 0;
    for (int l = 0; l < n_layers; ++l) {
        if (C[l] < 1 || C[l] > (1 << 15)) return false;      // 2C up to 65536
        const long long t = (2LL * C[l] + 63) / 64;
        tiles += t * t;
        if (tiles > (1LL << 30)) return false;
    }
    return true;
}
}  // namespace

size_t bn_full_workspace_bytes(int32_t n_layers, int32_t N, const int32_t *C)
{
    if (!bn_full_dims_ok(n_layers, N, C)) return 0;
    const Tunables tun(default_options());
    BnFullArgs a{};
    a.n_layers = n_layers; a.N = N; a.C = C;
    size_t all = 0, single = 0;
    {
        Plan plan; Arena arena(nullptr);
        plan_bn_full(plan, arena, tun, a, true);
        arena.take_tail(plan.tab.buf.size() + 16);
        all = arena.peak;
    }
    // a partial mask changes which products share a launch and hence their split-K scratch: the
    // largest single-layer plan on top covers that; the call itself checks the size in any case
    std::vector<uint8_t> mask(n_layers, 0);
    a.invert_mask = mask.data();
    for (int l = 0; l < n_layers; ++l) {
        bool seen = false;   // only a layer larger than all before it can raise the bound
        for (int q = 0; q < l; ++q) seen = seen || C[q] >= C[l];
        if (seen) continue;
        mask[l] = 1;
        Plan plan; Arena arena(nullptr);
        plan_bn_full(plan, arena, tun, a, true);
        single = std::max(single, arena.peak);
        mask[l] = 0;
    }
    return align_up(all + single + 4096, kAlign);
}

kfac_status bn_full_precondition(kfac_ctx *ctx, int32_t n_layers, int32_t N, const int32_t *C,
                                 const float *const *g_gamma, const float *const *g_beta, float decay, float lambda,
                                 float *const *F_ema, const uint8_t *invert_mask, float *const *F_inv, int32_t *info,
                                 float *const *out_gamma, float *const *out_beta)
{
    if (!ctx || !bn_full_dims_ok(n_layers, N, C)) return KFAC_ERR_INVALID;
    if (!g_gamma || !g_beta || !F_ema || !F_inv || !out_gamma || !out_beta) return KFAC_ERR_INVALID;
    if (!(decay >= 0.0f && decay < 1.0f) || !(lambda >= 0.0f) || !std::isfinite(lambda)) return KFAC_ERR_INVALID;
    for (int l = 0; l < n_layers; ++l) {
        if (!g_gamma[l] || !g_beta[l] || !F_ema[l] || !F_inv[l] || !out_gamma[l] || !out_beta[l]) return KFAC_ERR_INVALID;
        if (F_ema[l] == F_inv[l]) return KFAC_ERR_INVALID;
    }
    BnFullArgs a{n_layers, N, C, g_gamma, g_beta, decay, lambda, F_ema, invert_mask, F_inv, info, out_gamma, out_beta};
    Plan plan; Arena arena(ctx->ws);
    plan_bn_full(plan, arena, ctx->tun, a, false);
    return run_plan(ctx, plan, arena);
}

static kfac_status bn_reduce_call(int nhwc, kfac_ctx *ctx, int32_t n_layers, int32_t N, const int32_t *C,
                                    const int32_t *HW, const float *const *dy, const float *const *xhat,
                                    float *const *g_gamma, float *const *g_beta)
{
    if (!ctx || n_layers < 1 || n_layers > 65536 || N < 1 || !C || !HW) return KFAC_ERR_INVALID;
    if (!dy || !xhat || !g_gamma || !g_beta) return KFAC_ERR_INVALID;
    std::vector<BnReduceJob> jobs;
    long long wgs = 0;
    for (int l = 0; l < n_layers; ++l) {
        if (C[l] < 1 || C[l] > (1 << 24) || HW[l] < 1 || HW[l] > (1 << 24)) return KFAC_ERR_INVALID;
        if (!dy[l] || !xhat[l] || !g_gamma[l] || !g_beta[l]) return KFAC_ERR_INVALID;
        BnReduceJob J{};
        J.dy = dy[l]; J.xhat = xhat[l]; J.g_gamma = g_gamma[l]; J.g_beta = g_beta[l];
        J.C = C[l]; J.HW = HW[l];
        J.wg_start = (int)wgs;
        wgs += nhwc ? (long long)N * ((C[l] + 63) / 64) : ((long long)N * C[l] + 3) / 4;
        if (wgs > (1LL << 30)) return KFAC_ERR_INVALID;
        jobs.push_back(J);
    }
    Plan plan; Arena arena(ctx->ws);
    Launch Lc{};
    Lc.kind = L_BNRED;
    for (auto &J : jobs) Lc.bytes += 8.0 * N * J.C * J.HW + 8.0 * N * J.C;
    Lc.off_a = plan.tab.add(jobs.data(), jobs.size() * sizeof(BnReduceJob));
    Lc.n = n_layers;
    Lc.total_wgs = (int)wgs;
    Lc.cfg = N;
    Lc.dtype = nhwc;
    plan.launches.push_back(Lc);
    return run_plan(ctx, plan, arena);
}

kfac_status bn_unitwise_reduce_nchw(kfac_ctx *ctx, int32_t n_layers, int32_t N, const int32_t *C,
                                    const int32_t *HW, const float *const *dy, const float *const *xhat,
                                    float *const *g_gamma, float *const *g_beta)
{
    return bn_reduce_call(0, ctx, n_layers, N, C, HW, dy, xhat, g_gamma, g_beta);
}

kfac_status bn_unitwise_reduce_nhwc(kfac_ctx *ctx, int32_t n_layers, int32_t N, const int32_t *C,
                                    const int32_t *HW, const float *const *dy, const float *const *xhat,
                                    float *const *g_gamma, float *const *g_beta)
{
    return bn_reduce_call(1, ctx, n_layers, N, C, HW, dy, xhat, g_gamma, g_beta);
}

kfac_status kfac_staleness(kfac_ctx *ctx, int32_t n, const int32_t *dims, const float *const *X,
                           const float *const *X_m1, const float *const *X_m2, double *ratios)
{
    if (!ctx || n < 1 || n > 65536 || !dims || !X || !ratios) return KFAC_ERR_INVALID;
    Plan plan; Arena arena(ctx->ws);
    std::vector<StaleJob> jobs;
    long long wgs = 0;
    double bytes = 0;
    for (int i = 0; i < n; ++i) {
        if (dims[i] < 1 || dims[i] > (1 << 20) || !X[i]) return KFAC_ERR_INVALID;
        StaleJob J{};
        J.X = X[i];
        J.P = X_m1 ? X_m1[i] : nullptr;
        J.Q = X_m2 ? X_m2[i] : nullptr;
        if (J.P == J.X || J.Q == J.X) return KFAC_ERR_INVALID;   // a statistic is not its own predecessor
        J.n = (long long)dims[i] * dims[i];
        J.wgs = (int)((J.n + kStaleChunk - 1) / kStaleChunk);
        J.partial = (double *)arena.take((size_t)J.wgs * 4 * sizeof(double));
        J.out = ratios + 2 * i;
        J.wg_start = (int)wgs;
        wgs += J.wgs;
        if (wgs > (1LL << 30)) return KFAC_ERR_INVALID;
        bytes += 4.0 * J.n * (1 + (J.P ? 1 : 0) + (J.Q ? 1 : 0));
        jobs.push_back(J);
    }
    const size_t off = plan.tab.add(jobs.data(), jobs.size() * sizeof(StaleJob));
    for (int pass = 0; pass < 2; ++pass) {
        Launch L{};
        L.kind = L_STALE;
        L.off_a = off;
        L.n = n;
        L.total_wgs = pass == 0 ? (int)wgs : n;
        L.cfg = pass;
        L.bytes = pass == 0 ? bytes : 0.0;
        plan.launches.push_back(L);
    }
    return run_plan(ctx, plan, arena);
}

double kfac_lr_polynomial(double eta0, double e, double e_start, double e_end, double p_decay)
{
    if (!(e_end > e_start)) return NAN;
    if (e <= e_start) return eta0;
    if (e >= e_end) return 0.0;
    return eta0 * pow(1.0 - (e - e_start) / (e_end - e_start), p_decay);
}

double kfac_momentum_coupled(double m0, double eta0, double eta)
{
    if (eta0 == 0.0) return NAN;
    return m0 / eta0 * eta;
}

kfac_status kfac_update_weights(kfac_ctx *ctx, int32_t n_layers, const kfac_layer *L, const float *const *U,
                                float eta, float momentum, int32_t rescale, float eps, float *const *W,
                                float *const *W_prev)
{
    if (!ctx || n_layers < 1 || n_layers > 65536 || !L || !U || !W || !W_prev) return KFAC_ERR_INVALID;
    if (!std::isfinite(eta) || !std::isfinite(momentum) || !(eps >= 0.f) || !std::isfinite(eps)) return KFAC_ERR_INVALID;
    Plan plan; Arena arena(ctx->ws);
    std::vector<UpdateJob> jobs;
    long long wgs = 0;
    double bytes = 0;
    for (int l = 0; l < n_layers; ++l) {
        int dA, dG;
        if (!layer_ok(L[l], &dA, &dG, nullptr, nullptr)) return KFAC_ERR_INVALID;
        if (!U[l] || !W[l] || !W_prev[l]) return KFAC_ERR_INVALID;
        const size_t sz = (size_t)dA * dG * sizeof(float);
        auto overlap = [&](const void *a, const void *b) { return (const char *)a < (const char *)b + sz && (const char *)b < (const char *)a + sz; };
        if (overlap(U[l], W[l]) || overlap(U[l], W_prev[l]) || overlap(W[l], W_prev[l])) return KFAC_ERR_INVALID;
        UpdateJob J{};
        J.W = W[l]; J.W_prev = W_prev[l]; J.U = U[l];
        J.n = (long long)dA * dG;
        J.d_out = dG;
        J.wgs = (int)((J.n + kUpdateChunk - 1) / kUpdateChunk);
        if (rescale) {
            J.partial = (double *)arena.take((size_t)J.wgs * sizeof(double));
            J.scale = (float *)arena.take(sizeof(float));
        }
        J.wg_start = (int)wgs;
        wgs += J.wgs;
        if (wgs > (1LL << 30)) return KFAC_ERR_INVALID;
        bytes += 4.0 * J.n;
        jobs.push_back(J);
    }
    const size_t off = plan.tab.add(jobs.data(), jobs.size() * sizeof(UpdateJob));
    for (int pass = 0; pass < (rescale ? 3 : 1); ++pass) {
        Launch Lc{};
        Lc.kind = L_UPDATE;
        Lc.off_a = off;
        Lc.n = n_layers;
        Lc.total_wgs = (int)wgs;
        Lc.cfg = pass;
        Lc.f0 = pass == 1 ? eps : eta;
        Lc.f1 = momentum;
        Lc.bytes = pass == 0 ? 5.0 * bytes : (pass == 2 ? 2.0 * bytes : 0.0);
        plan.launches.push_back(Lc);
    }
    return run_plan(ctx, plan, arena);
}

kfac_status kfac_nhwc_to_nchw(kfac_ctx *ctx, int32_t n_layers, const kfac_layer *L, int32_t which, kfac_dtype type,
                              const void *const *src, void *const *dst)
{
    if (!ctx || !layers_ok(L, n_layers) || !src || !dst) return KFAC_ERR_INVALID;
    if ((which != 0 && which != 1) || (type != KFAC_F32 && type != KFAC_BF16)) return KFAC_ERR_INVALID;
    const int esize = type == KFAC_F32 ? 4 : 2;
    std::vector<LayoutJob> jobs;
    long long wgs = 0;
    double bytes = 0;
    for (int l = 0; l < n_layers; ++l) {
        if (!src[l]) continue;
        if (!dst[l]) return KFAC_ERR_INVALID;
        int h, w;
        layer_ok(L[l], nullptr, nullptr, &h, &w);
        LayoutJob J{};
        J.src = src[l]; J.dst = dst[l];
        J.N = L[l].N;
        J.C = which == 0 ? L[l].c_in : L[l].c_out;
        J.HW = which == 0 ? L[l].h_in * L[l].w_in : h * w;
        const size_t sz = (size_t)J.N * J.C * J.HW * esize;
        if ((const char *)J.src < (const char *)J.dst + sz && (const char *)J.dst < (const char *)J.src + sz)
            return KFAC_ERR_INVALID;   // the conversion is not done in place
        J.tiles_c = (J.C + 63) / 64;
        J.tiles_hw = (J.HW + 63) / 64;
        J.wg_start = (int)wgs;
        wgs += (long long)J.N * J.tiles_c * J.tiles_hw;
        if (wgs > (1LL << 30)) return KFAC_ERR_INVALID;
        bytes += 2.0 * sz;
        jobs.push_back(J);
    }
    if (jobs.empty()) return KFAC_OK;
    Plan plan; Arena arena(ctx->ws);
    Launch Lc{};
    Lc.kind = L_LAYOUT;
    Lc.off_a = plan.tab.add(jobs.data(), jobs.size() * sizeof(LayoutJob));
    Lc.n = (int)jobs.size();
    Lc.total_wgs = (int)wgs;
    Lc.cfg = esize;
    Lc.bytes = bytes;
    plan.launches.push_back(Lc);
    return run_plan(ctx, plan, arena);
}

size_t kfac_packed_elems(int32_t n, const int32_t *dims)
{
    if (n < 1 || !dims) return 0;
    size_t total = 0;
    for (int i = 0; i < n; ++i) {
        if (dims[i] < 1 || dims[i] > (1 << 20)) return 0;
        total += (size_t)dims[i] * ((size_t)dims[i] + 1) / 2;
    }
    return total;
}

static kfac_status pack_call(kfac_ctx *ctx, int32_t n, const int32_t *dims, const float *const *X, kfac_dtype type,
                             void *packed, int unpack)
{
    if (!ctx || n < 1 || n > 65536 || !dims || !X || !packed) return KFAC_ERR_INVALID;
    if (type != KFAC_F32 && type != KFAC_BF16) return KFAC_ERR_INVALID;
    const size_t total = kfac_packed_elems(n, dims);
    if (total == 0) return KFAC_ERR_INVALID;
    const size_t esize = type == KFAC_BF16 ? 2 : 4;
    const char *p0 = (const char *)packed, *p1 = p0 + total * esize;
    Plan plan; Arena arena(ctx->ws);
    std::vector<PackJob> jobs;
    long long wgs = 0, off = 0;
    for (int i = 0; i < n; ++i) {
        if (!X[i]) return KFAC_ERR_INVALID;
        const char *x0 = (const char *)X[i], *x1 = x0 + (size_t)dims[i] * dims[i] * sizeof(float);
        if (x0 < p1 && p0 < x1) return KFAC_ERR_INVALID;   // a matrix overlaps the packed buffer
        PackJob J{};
        J.X = X[i];
        J.off = off;
        J.d = dims[i];
        J.tiles = (dims[i] + 63) / 64;
        J.wg_start = (int)wgs;
        const long long tri = (long long)dims[i] * (dims[i] + 1) / 2;
        wgs += unpack ? (long long)J.tiles * (J.tiles + 1) / 2 : (tri + kPackChunk - 1) / kPackChunk;
        off += tri;
        if (wgs > (1LL << 30)) return KFAC_ERR_INVALID;
        jobs.push_back(J);
    }
    Launch L{};
    L.kind = L_PACK;
    L.off_a = plan.tab.add(jobs.data(), jobs.size() * sizeof(PackJob));
    L.n = n;
    L.total_wgs = (int)wgs;
    L.cfg = unpack;
    L.dtype = type == KFAC_BF16 ? 1 : 0;
    L.p0 = packed;
    // packing reads and writes the triangle; unpacking reads it and writes the whole matrix
    double full = 0;
    for (int i = 0; i < n; ++i) full += 4.0 * dims[i] * dims[i];
    L.bytes = unpack ? (double)total * esize + full : (double)total * (4.0 + esize);
    plan.launches.push_back(L);
    return run_plan(ctx, plan, arena);
}

kfac_status kfac_pack_upper(kfac_ctx *ctx, int32_t n, const int32_t *dims, const float *const *X,
                            kfac_dtype type, void *packed)
{
    return pack_call(ctx, n, dims, X, type, packed, 0);
}

kfac_status kfac_unpack_upper(kfac_ctx *ctx, int32_t n, const int32_t *dims, kfac_dtype type,
                              const void *packed, float *const *X)
{
    return pack_call(ctx, n, dims, (const float *const *)X, type, const_cast<void *>(packed), 1);
}

int32_t kfac_next_interval(int32_t similar_to_last, int32_t similar_to_before_last, int32_t delta_m1,
                           int32_t delta_m2)
{
    if (delta_m1 < 1 || delta_m2 < 1) return 0;
    if (!similar_to_last) return std::max(1, delta_m1 / 2);
    if (!similar_to_before_last) return delta_m1;
    const long long sum = (long long)delta_m1 + delta_m2;
    return (int32_t)std::min<long long>(sum, INT32_MAX);
}

void kfac_refresh_init(kfac_refresh_state *s, int32_t n)
{
    if (!s) return;
    for (int32_t i = 0; i < n; ++i) { s[i].t_next = 1; s[i].delta = 1; s[i].delta_m1 = 1; }
}

int32_t kfac_refresh_due(const kfac_refresh_state *s, int32_t t) { return s && t == s->t_next ? 1 : 0; }

void kfac_refresh_advance(kfac_refresh_state *s, double ratio_m1, double ratio_m2, double alpha)
{
    if (!s) return;
    // (a NaN ratio compares false: not similar)
    const int32_t next = kfac_next_interval(ratio_m1 < alpha, ratio_m2 < alpha, std::max(1, s->delta),
                                            std::max(1, s->delta_m1));
    s->delta_m1 = s->delta;
    s->delta = next;
    const long long t = (long long)s->t_next + next;
    s->t_next = (int32_t)std::min<long long>(t, INT32_MAX);
}

}  // extern "C"
