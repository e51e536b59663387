// C ABI of the solver: contexts, graph loading (validate, reorder, cut into
// octiles, bitmap-pack, upload), job lists and kernel launches.
#include <hip/hip_runtime_api.h>

#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>
#include <numeric>
#include <stdexcept>
#include <string>
#include <system_error>
#include <thread>
#include <vector>

#include "../../include/mgk.h"
#include "mgk_internal.h"
#include "mgk_launch.h"
#include "mgk_reorder.h"

namespace {

constexpr int kTile = 8;

struct JobBin {
    int64_t first = 0;   // index of the bin's first job in the job array
    int64_t count = 0;
    size_t lds_bytes = 0;
    int waves = 0, ept = 0;
    int chunks = 0;            // > 0: register-resident solver with this many inner chunks
    int sell_regs = 0;         // > 0: owner-computes solver with this many entry registers per lane
    bool atomic_rows = false;  // an inner graph has a row longer than one lane group
    bool swapped = false;      // outer graphs come from batch Y, inner from X
};

struct JobList {
    MgkJob* dev = nullptr;
    int64_t n = 0;
    std::vector<JobBin> bins;
    // pairs whose vectors do not fit on chip: [outer graph from X / from Y][sparse / dense tile path]
    std::vector<MgkLargePair> large[2][2];
};

// growable device allocation owned by a context
struct DevBuf {
    void* p = nullptr;
    size_t cap = 0;
};

}  // namespace

struct mgk_batch {
    mgk_ctx* owner = nullptr;
    int32_t n_graphs = 0;
    int64_t n_vertices = 0, nnz = 0, n_tiles = 0, n_offdiag = 0;
    bool weighted = false;
    int label_dim = 1;
    double label_mean = 0.0;
    // host copies
    std::vector<MgkGraphDesc> graphs;
    std::vector<MgkTile> tiles;
    std::vector<float> w, e;
    std::vector<int32_t> perm;     // [n_vertices], perm[voff + old] = new
    std::vector<int64_t> vtx_off;  // [G+1]
    std::vector<MgkSellDesc> sell_desc;   // per graph, for the planner
    // device
    void* blob = nullptr;
    MgkBatchDev dev{};
    JobList gram_jobs;
    int gram_jobs_waves = 0;       // waves_per_pair setting the list was built for
    int gram_jobs_max_iter = 0;    // max_iter setting the list was built for
    int gram_jobs_limit = 0;       // on-chip limit the list was built for
    int gram_jobs_tile_path = 0;   // tile path setting the list was built for
    int gram_jobs_cache = 0;       // product-cache setting the list was built for
    int gram_jobs_sorted = 0;      // schedule setting the list was built for
    int gram_jobs_attr_dim = -1;   // label attributes of the edge kernel it was built for (LDS plan)
};

struct mgk_ctx {
    int device = 0;
    std::string err;
    float q = 0.05f, h = 1.0f, length_scale = 1.0f, ke_const = 1.0f, rtol = 1e-6f;
    int edge_kernel = MGK_EK_CONST;
    int label_dim = 1;                          // attributes the edge kernel reads
    float attr_ls[MGK_MAX_LABEL_DIM] = {1.f, 1.f, 1.f, 1.f};  // length scales of kron_se / rconv_se
    float poly_c[MGK_POLY_MAX_COEF] = {};
    float poly_rho = 1.f;
    int max_iter = 0;
    int tile_path = MGK_TILE_AUTO;
    int waves = 0;
    int onchip_limit = MGK_SMALL_MAX_N;  // largest n n' given to the on-chip solver
    int product_cache = 1;      // small pairs keep their matrix entries in registers (2, 3: one of the two kernels only)
    int cost_sorted = 1;        // expensive pairs first inside a launch
    int row_staging = 1;        // global-memory sparse product stages rows of p in LDS
    JobList pair_jobs;          // reused by mgk_pairs
    int64_t pair_jobs_cap = 0;
    hipStream_t pair_jobs_stream = nullptr;
    bool pair_jobs_busy = false;
    hipStream_t fixed_jobs_stream = nullptr;   // last mgk_pairs_noalloc call of this context
    bool fixed_jobs_busy = false;
    // scratch of the global-memory solver
    DevBuf exp_outer[2], exp_inner[2];  // expanded entry lists of batch X / batch Y
    DevBuf dense_tiles[2][3];           // dense 8x8 expansions (weight, label, log2 weight)
    DevBuf vec, lpairs, lstate, lactive, nodal_off, diag;
    int* active_host = nullptr;         // pinned: {pairs still iterating, most iterations needed}
    void* pin = nullptr;                // pinned staging of the pair records of a call
    size_t pin_cap = 0;
    hipEvent_t pin_event = nullptr;     // recorded after the last copy out of `pin`
    bool pin_busy = false;
    int large_iter_guess = 12;          // iterations the last call of the global-memory solver needed
    std::string launch_log;             // kernels the last solve call enqueued, one line each
};

namespace {

mgk_status fail(mgk_ctx* ctx, mgk_status st, const char* fmt, ...) noexcept {
    if (ctx) {
        char buf[512];
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(buf, sizeof buf, fmt, ap);
        va_end(ap);
        try { ctx->err = buf; } catch (...) { ctx->err.clear(); }   // capacity is reserved at creation
    }
    return st;
}

void log_launch(mgk_ctx* ctx, const char* fmt, ...) {
    char buf[256];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    ctx->launch_log += buf;
    ctx->launch_log += '\n';
}

#define MGK_HIP(ctx, call)                                                              \
    do {                                                                                \
        hipError_t e_ = (call);                                                         \
        if (e_ != hipSuccess)                                                           \
            return fail(ctx, MGK_EDEVICE, "%s failed: %s", #call, hipGetErrorString(e_)); \
    } while (0)

// Runs `body` and turns any C++ exception into a status, so that nothing unwinds
// across the C ABI.  The message is stored without allocating when memory is short.
template <class F>
mgk_status guarded(mgk_ctx* ctx, F&& body) noexcept {
    mgk_status st = MGK_EINVAL;
    const char* what = "unexpected exception";
    try {
        return body();
    } catch (const std::bad_alloc&) {
        st = MGK_ENOMEM;
        what = "out of host memory";
    } catch (const std::length_error&) {
        st = MGK_ELIMIT;
        what = "request exceeds the largest host array";
    } catch (const std::system_error&) {
        st = MGK_ENOMEM;
        what = "could not start a worker thread";
    } catch (...) {
    }
    if (ctx) {
        try { ctx->err = what; } catch (...) { ctx->err.clear(); }
    }
    return st;
}

// Worker threads that are always joined, also when starting one of them throws.
struct JoiningThreads {
    std::vector<std::thread> t;
    ~JoiningThreads() { join(); }
    void join() {
        for (std::thread& th : t)
            if (th.joinable()) th.join();
    }
};

template <class T>
size_t append_bytes(std::vector<char>& blob, const std::vector<T>& v) {
    size_t off = (blob.size() + 255) & ~(size_t)255;
    blob.resize(off + std::max<size_t>(v.size() * sizeof(T), 16));
    if (!v.empty()) memcpy(blob.data() + off, v.data(), v.size() * sizeof(T));
    return off;
}

// Contiguous division of the rows of a graph among `waves` wavefronts for the
// register-resident solver: bounds[w] .. bounds[w+1] are wavefront w's rows.  A row of
// deg nonzeros costs about 4 deg + 9 wave instructions of an XMV (two inner chunks: an
// address add and a multiply-add per nonzero and chunk, the row sums and the store at its
// end); the largest cost of a wavefront is made as small as whole rows allow (bisection
// on the bound, rows filled in greedily).  Returns the most nonzeros a wavefront gets.
int balanced_split(const std::vector<int32_t>& deg, int n, int waves, int32_t* bounds) {
    auto row_cost = [&](int i) { return (int64_t)4 * deg[i] + 9; };
    int64_t lo = 0, hi = 0;
    for (int i = 0; i < n; ++i) { lo = std::max(lo, row_cost(i)); hi += row_cost(i); }
    auto parts_needed = [&](int64_t bound) {
        int parts = 1;
        int64_t cur = 0;
        for (int i = 0; i < n; ++i) {
            if (cur + row_cost(i) > bound) { ++parts; cur = row_cost(i); } else cur += row_cost(i);
        }
        return parts;
    };
    while (lo < hi) {
        const int64_t mid = (lo + hi) / 2;
        if (parts_needed(mid) <= waves) hi = mid; else lo = mid + 1;
    }
    int w = 0, longest = 0, run = 0;
    int64_t cur = 0;
    bounds[0] = 0;
    for (int i = 0; i < n; ++i) {
        if (cur + row_cost(i) > lo) { bounds[++w] = i; cur = 0; run = 0; }
        cur += row_cost(i);
        run += deg[i];
        longest = std::max(longest, run);
    }
    while (w < waves) bounds[++w] = n;
    return longest;
}

// attributes per edge label that the edge kernel reads (0 for the kernels on plain
// scalar labels); the streaming on-chip solver keeps them in LDS for the outer graph
int attr_dim_of(const mgk_ctx* ctx) {
    return ctx->edge_kernel == MGK_EK_KRON_SE || ctx->edge_kernel == MGK_EK_RCONV_SE ? ctx->label_dim : 0;
}

// the batches must carry the number of label attributes the edge kernel reads
mgk_status check_label_dim(mgk_ctx* ctx, const mgk_batch* X, const mgk_batch* Y) {
    if (attr_dim_of(ctx) == 0) return MGK_OK;
    if (X->label_dim != ctx->label_dim || Y->label_dim != ctx->label_dim)
        return fail(ctx, MGK_ESTATE, "edge kernel reads %d label attributes, the batches hold %d and %d",
                    ctx->label_dim, X->label_dim, Y->label_dim);
    return MGK_OK;
}

MgkParams make_params(const mgk_ctx* ctx, const mgk_batch* X) {
    MgkParams p{};
    p.q = ctx->q;
    p.h = ctx->h;
    const double log2e = 1.4426950408889634;
    const double alpha = 1.0 / (2.0 * (double)ctx->length_scale * (double)ctx->length_scale);
    p.e_scale = (float)std::sqrt(alpha * log2e);  // exp(-a d^2) = exp2(-(d sqrt(a log2 e))^2)
    p.e_shift = (float)X->label_mean;
    if (ctx->edge_kernel == MGK_EK_POLY) p.e_scale = 1.0f / ctx->poly_rho;
    p.label_dim = ctx->edge_kernel == MGK_EK_KRON_SE || ctx->edge_kernel == MGK_EK_RCONV_SE ? ctx->label_dim : 1;
    for (int a = 0; a < MGK_MAX_LABEL_DIM; ++a) {
        const double l = ctx->attr_ls[ctx->edge_kernel == MGK_EK_RCONV_SE ? 0 : a];
        p.attr_scale[a] = (float)std::sqrt(log2e / (2.0 * l * l));
    }
    for (int i = 0; i < MGK_POLY_MAX_COEF; ++i) p.poly_c[i] = ctx->poly_c[i];
    p.ke_const = ctx->ke_const;
    p.rtol2 = ctx->rtol * ctx->rtol;
    p.max_iter = ctx->max_iter;
    p.edge_kernel = ctx->edge_kernel;
    return p;
}

// Launch shapes of the on-chip solver: `waves` wavefronts per pair, `ept`
// vector elements per thread; a pair fits when n n' <= waves * 64 * ept.
struct SmallConfig { int waves, ept; };
const SmallConfig kAutoConfigs[] = {{1, 4}, {2, 4}, {4, 4}, {4, 6}, {4, 8}, {4, 10}, {4, 12}, {4, 14}, {4, 16}, {8, 12}, {8, 16}, {16, 10}, {16, 12}, {16, 16}};
const int kEpts[] = {4, 8, 12, 16};

// Orientation, launch shape and cost of one pair for the on-chip solver.  The
// inner graph's nonzeros are spread over lanes in chunks of 64, the outer
// graph's are streamed, so the work is z_outer * ceil(z_inner / 64) wave
// iterations.
struct PairPlan {
    bool swap = false;   // true: Y's graph is the outer one
    bool atomic_rows = false;
    int64_t cost = 0;
    int64_t lds_words = 0;
    int waves = 0, ept = 0;  // 0: does not fit
    int chunks = 0;          // > 0: register-resident solver
    int sell_regs = 0;       // > 0: owner-computes solver
};

// Register-resident solver for (outer o, inner i) with `waves` wavefronts: every
// wavefront's run of outer rows must fit the unrolled loop, the inner layout the
// chunk registers, the vectors the register blocks.  Returns the cost in wave
// instructions of one iteration, or -1 if the pair does not fit.
int64_t regs_cost(const MgkGraphDesc& o, const MgkGraphDesc& i, int waves) {
    const int chunks = std::max(1, i.lane_len / 64);
    if (chunks > MGK_REGS_MAX_CHUNKS || i.max_deg > MGK_REGS_MAX_DEG) return -1;
    const int smax = waves == 4 ? MGK_REGS_SMAX_W4 : MGK_REGS_SMAX_W8;
    const int run = waves == 4 ? (o.regs_runs & 0xffff) : (int)((uint32_t)o.regs_runs >> 16);
    if (run > smax) return -1;
    const int64_t N = (int64_t)o.n * i.n;
    const int64_t ept = std::max<int64_t>(1, (N + waves * 64 - 1) / (waves * 64));
    // register blocks that keep four wavefronts per SIMD resident
    if (ept > MGK_REGS_MAX_EPT) return -1;
    return (int64_t)o.nnz * (2 * chunks) + (int64_t)o.n * (1 + 4 * chunks) +
           (int64_t)waves * (8 * ept + 45);
}

// Owner-computes solver for (outer o, inner i): the cheapest launch shape that holds the
// pair.  Cost in wave instructions of one iteration: the entries of the most loaded
// wavefront (a gather, weighted by its bank conflicts, and a multiply-add each), the
// vector part per slot, the three workgroup sums, and the share of the compute unit the
// workgroup occupies.  Returns -1 when no shape fits.
int64_t sell_cost(const MgkSellDesc& o, const MgkSellDesc& i, int* waves, int* ept, int* regs) {
    int64_t best = -1;
    for (int w = 4; w <= 16; w *= 2) {
        int32_t slots = 0, executed = 0;
        const int32_t need = mgk_sell_need(o, i, w, &slots, &executed);
        for (const MgkSellShape& sh : kMgkSellShapes)
            if (sh.waves == w && sh.ept >= slots && sh.regs >= need) {
                const int64_t c = (int64_t)executed * 4 + (int64_t)w * (13 * slots + 45);
                if (best < 0 || c < best) {
                    best = c;
                    *waves = w;
                    *ept = sh.ept;
                    *regs = sh.regs;
                }
                break;   // shapes of a workgroup size are listed smallest first
            }
    }
    return best;
}

// cache: 0 entries regenerated in every product; 1 (and 2) kept in registers by the kernel
// in which a wavefront owns rows of the outer graph; 3 by the owner-computes kernel where
// a pair fits it, else as 1
PairPlan plan_pair(const MgkGraphDesc& a, const MgkGraphDesc& b, const MgkSellDesc* sa, const MgkSellDesc* sb,
                   bool may_swap, int forced_waves, int onchip_limit, int cache, int attr_dim) {
    const bool product_cache = cache != 0;
    // wave iterations of one XMV: outer nonzeros x 64-lane chunks of the inner layout
    auto passes = [](const MgkGraphDesc& o, const MgkGraphDesc& i) {
        return (int64_t)o.nnz * (i.lane_len / 64) + 2 * (int64_t)o.n * (i.lane_len / 64);
    };
    PairPlan pl;
    const int64_t keep = passes(a, b), swp = passes(b, a);
    const bool keep_atomic = b.max_deg > MGK_LANE_GROUP, swp_atomic = a.max_deg > MGK_LANE_GROUP;
    pl.swap = may_swap && (keep_atomic != swp_atomic ? keep_atomic : swp < keep);
    pl.atomic_rows = pl.swap ? swp_atomic : keep_atomic;
    const int64_t N = (int64_t)a.n * b.n;
    pl.cost = (pl.swap ? swp : keep) * 64 + 16 * N;
    if (N > MGK_SMALL_MAX_N || N > onchip_limit) return pl;
    if (cache == 3 && forced_waves == 0 && attr_dim == 0 && sa && sb &&
        mgk_sell_ok(*sa) && mgk_sell_ok(*sb)) {
        int64_t best = -1;
        for (int sw = 0; sw < (may_swap ? 2 : 1); ++sw) {
            int w = 0, ept = 0, regs = 0;
            const int64_t c = sw ? sell_cost(*sb, *sa, &w, &ept, &regs) : sell_cost(*sa, *sb, &w, &ept, &regs);
            if (c >= 0 && (best < 0 || c < best)) {
                best = c;
                pl.waves = w;
                pl.ept = ept;
                pl.sell_regs = regs;
                pl.swap = sw != 0;
            }
        }
        if (best >= 0) {
            const MgkGraphDesc& o = pl.swap ? b : a;
            const MgkGraphDesc& i = pl.swap ? a : b;
            pl.atomic_rows = false;
            pl.chunks = 0;
            pl.cost = best * 16 + 16 * N;
            pl.lds_words = mgk_sell_plan(o.n, i.n, pl.waves, pl.ept).total;
            return pl;
        }
    }
    if (product_cache && forced_waves == 0) {
        int64_t best = -1;
        for (int w = 4; w <= 8; w *= 2)
            for (int sw = 0; sw < (may_swap ? 2 : 1); ++sw) {
                const int64_t c = sw ? regs_cost(b, a, w) : regs_cost(a, b, w);
                if (c >= 0 && (best < 0 || c < best)) { best = c; pl.waves = w; pl.swap = sw != 0; }
            }
        if (best >= 0) {
            const MgkGraphDesc& o = pl.swap ? b : a;
            const MgkGraphDesc& i = pl.swap ? a : b;
            pl.atomic_rows = false;
            pl.ept = (int)std::max<int64_t>(1, (N + pl.waves * 64 - 1) / (pl.waves * 64));
            pl.chunks = std::max(1, i.lane_len / 64);
            pl.cost = best * 16 + 16 * N;
            pl.lds_words = mgk_regs_plan(o.n, i.n, pl.waves, pl.ept).total;
            return pl;
        }
    }
    if (forced_waves > 0) {  // requested workgroup size, doubled until the pair fits
        for (int w = forced_waves; w <= 16 && pl.waves == 0; w *= 2)
            for (int e : kEpts)
                if ((int64_t)w * 64 * e >= N) { pl.waves = w; pl.ept = e; break; }
    } else {
        for (const SmallConfig& c : kAutoConfigs)
            if ((int64_t)c.waves * 64 * c.ept >= N) { pl.waves = c.waves; pl.ept = c.ept; break; }
    }
    if (pl.waves == 0) return pl;
    const MgkGraphDesc& o = pl.swap ? b : a;
    const MgkGraphDesc& i = pl.swap ? a : b;
    pl.lds_words = mgk_small_plan(o.n, i.n, o.nnz, i.lane_len, o.n_tiles, i.n_tiles, pl.waves, pl.ept, attr_dim).total;
    if (pl.lds_words * 4 > MGK_LDS_LIMIT_BYTES) pl.waves = pl.ept = 0;
    return pl;
}

struct HostJob {
    MgkJob job;
    int64_t cost;
    int32_t lds_words;
    int16_t waves, ept, chunks;
    int16_t sell_regs = 0;
    bool atomic_rows, swapped;
};

// A launch shape with few jobs costs more in launch and drain time than its pairs
// gain from the exact fit: such jobs move to the closest larger shape that can run
// them (same solver and workgroup size, at least as many elements per thread and
// inner chunks).  Only the vector blocks grow, so the LDS need grows by the
// difference of the padded vector lengths.
constexpr int64_t kMinJobsPerLaunch = 4096;

void merge_small_shapes(std::vector<HostJob>& jobs) {
    struct Shape { int waves, ept, chunks, sell_regs; bool atomic_rows, swapped; int64_t count; };
    auto same = [](const Shape& s, const HostJob& j) {
        return s.waves == j.waves && s.ept == j.ept && s.chunks == j.chunks && s.sell_regs == j.sell_regs &&
               s.atomic_rows == j.atomic_rows && s.swapped == j.swapped;
    };
    std::vector<Shape> frozen;   // shapes whose jobs would outgrow LDS in the larger shape
    for (int round = 0; round < 64; ++round) {
        std::vector<Shape> shapes;
        for (const HostJob& j : jobs) {
            auto it = std::find_if(shapes.begin(), shapes.end(), [&](const Shape& s) { return same(s, j); });
            if (it == shapes.end()) shapes.push_back({j.waves, j.ept, j.chunks, j.sell_regs, j.atomic_rows, j.swapped, 1});
            else it->count++;
        }
        // smallest shape below the threshold that has somewhere to go
        const Shape* from = nullptr;
        const Shape* to = nullptr;
        for (const Shape& a : shapes) {
            if (a.count >= kMinJobsPerLaunch) continue;
            if (std::any_of(frozen.begin(), frozen.end(), [&](const Shape& f) {
                    return f.waves == a.waves && f.ept == a.ept && f.chunks == a.chunks && f.sell_regs == a.sell_regs &&
                           f.atomic_rows == a.atomic_rows && f.swapped == a.swapped; }))
                continue;
            const Shape* best = nullptr;
            for (const Shape& b : shapes) {
                if (&a == &b || a.waves != b.waves || a.atomic_rows != b.atomic_rows || a.swapped != b.swapped ||
                    (a.chunks > 0) != (b.chunks > 0) || b.chunks < a.chunks || b.ept < a.ept ||
                    (a.sell_regs > 0) != (b.sell_regs > 0) || b.sell_regs < a.sell_regs)
                    continue;
                if (!best || b.ept * 4 + b.chunks + b.sell_regs < best->ept * 4 + best->chunks + best->sell_regs) best = &b;
            }
            if (best && (!from || a.ept * 4 + a.chunks < from->ept * 4 + from->chunks)) { from = &a; to = best; }
        }
        if (!from) return;
        // padded vectors in the LDS plan of each solver (the owner-computes one also has a
        // schedule word per wavefront and slot; 4 words of alignment slack)
        const int vectors = from->sell_regs > 0 ? 3 : from->chunks > 0 ? 4 : 2;
        const int extra = from->sell_regs > 0 ? from->waves * (to->ept - from->ept) + 4 : 0;
        bool fits = true;
        for (const HostJob& j : jobs)
            if (same(*from, j) &&
                ((int64_t)j.lds_words + vectors * j.waves * 64 * (to->ept - j.ept) + extra) * 4 > MGK_LDS_LIMIT_BYTES)
                fits = false;
        if (!fits) { frozen.push_back(*from); continue; }
        for (HostJob& j : jobs)
            if (same(*from, j)) {
                j.lds_words += vectors * j.waves * 64 * (to->ept - j.ept) + extra;
                j.ept = (int16_t)to->ept;
                j.chunks = (int16_t)to->chunks;
                j.sell_regs = (int16_t)to->sell_regs;
            }
    }
}

// `fixed`: the job array is storage the caller provides (`out.dev` set, *capacity jobs);
// nothing is allocated or freed then.
mgk_status build_job_list(mgk_ctx* ctx, std::vector<HostJob>& jobs, JobList& out,
                          hipStream_t stream, int64_t* capacity, bool fixed = false) {
    merge_small_shapes(jobs);
    // group by launch shape (largest first), inside a group big pairs start first
    const bool by_cost = ctx->cost_sorted != 0;
    std::stable_sort(jobs.begin(), jobs.end(), [by_cost](const HostJob& a, const HostJob& b) {
        const int ka = a.waves * 64 * a.ept, kb = b.waves * 64 * b.ept;
        if (ka != kb) return ka > kb;
        if (a.waves != b.waves) return a.waves > b.waves;
        if (a.chunks != b.chunks) return a.chunks > b.chunks;
        if (a.sell_regs != b.sell_regs) return a.sell_regs > b.sell_regs;
        if (a.atomic_rows != b.atomic_rows) return a.atomic_rows;
        if (a.swapped != b.swapped) return b.swapped;
        return by_cost && a.cost > b.cost;
    });
    out.bins.clear();
    out.n = (int64_t)jobs.size();
    std::vector<MgkJob> flat(jobs.size());
    for (size_t k = 0; k < jobs.size(); ++k) {
        flat[k] = jobs[k].job;
        if (out.bins.empty() || jobs[k].waves != out.bins.back().waves ||
            jobs[k].ept != out.bins.back().ept || jobs[k].chunks != out.bins.back().chunks ||
            jobs[k].sell_regs != out.bins.back().sell_regs ||
            jobs[k].atomic_rows != out.bins.back().atomic_rows ||
            jobs[k].swapped != out.bins.back().swapped) {
            JobBin b;
            b.first = (int64_t)k;
            b.waves = jobs[k].waves;
            b.ept = jobs[k].ept;
            b.chunks = jobs[k].chunks;
            b.sell_regs = jobs[k].sell_regs;
            b.atomic_rows = jobs[k].atomic_rows;
            b.swapped = jobs[k].swapped;
            out.bins.push_back(b);
        }
        JobBin& b = out.bins.back();
        b.count++;
        b.lds_bytes = std::max(b.lds_bytes, (size_t)jobs[k].lds_words * 4);
    }
    if (fixed) {
        if (out.n > *capacity) return fail(ctx, MGK_ELIMIT, "job list of %lld pairs exceeds the fixed storage of %lld",
                                           (long long)out.n, (long long)*capacity);
    } else if (capacity == nullptr || *capacity < out.n) {
        if (out.dev) MGK_HIP(ctx, hipFree(out.dev));
        out.dev = nullptr;
        const int64_t cap = std::max<int64_t>(out.n, 1);
        MGK_HIP(ctx, hipMalloc((void**)&out.dev, (size_t)cap * sizeof(MgkJob)));
        if (capacity) *capacity = cap;
    }
    if (out.n) {
        MGK_HIP(ctx, hipMemcpyAsync(out.dev, flat.data(), (size_t)out.n * sizeof(MgkJob),
                                    hipMemcpyHostToDevice, stream));
        MGK_HIP(ctx, hipStreamSynchronize(stream));  // `flat` is pageable and dies here
    }
    return MGK_OK;
}

mgk_status ensure(mgk_ctx* ctx, DevBuf& b, size_t bytes) {
    if (bytes <= b.cap) return MGK_OK;
    if (b.p) MGK_HIP(ctx, hipFree(b.p));
    b.p = nullptr;
    b.cap = 0;
    hipError_t e = hipMalloc(&b.p, bytes);
    if (e != hipSuccess)
        return fail(ctx, MGK_ENOMEM, "device allocation of %zu bytes failed: %s", bytes, hipGetErrorString(e));
    b.cap = bytes;
    return MGK_OK;
}

// Tile-pair primitive for a pair in the global-memory solver (Section IV-B,
// "hybrid dense-sparse"): the dense primitive evaluates all 4096 products of a
// tile pair, the sparse one only nnz * nnz' of them but pays gathers and row
// sums; the dense one wins when both graphs' tiles are well filled.
constexpr int kDenseMinNnzPerTile = 53;   // measured crossover on 256-vertex graphs: density 0.82

bool use_dense_tiles(const mgk_ctx* ctx, const MgkGraphDesc& a, const MgkGraphDesc& b) {
    if (ctx->edge_kernel == MGK_EK_KRON_SE || ctx->edge_kernel == MGK_EK_RCONV_SE) return false;
    if (ctx->tile_path == MGK_TILE_DENSE) return true;
    if (ctx->tile_path == MGK_TILE_SPARSE || ctx->tile_path == MGK_TILE_SPARSE_GATHER) return false;
    return a.n_tiles > 0 && b.n_tiles > 0 &&
           (int64_t)a.nnz >= (int64_t)kDenseMinNnzPerTile * a.n_tiles &&
           (int64_t)b.nnz >= (int64_t)kDenseMinNnzPerTile * b.n_tiles;
}

// Plan of one pair for the global-memory solver (any size).
MgkLargePair plan_large(const MgkGraphDesc& a, const MgkGraphDesc& b, int32_t ia, int32_t ib, bool* swap,
                        int max_iter_param) {
    auto passes = [](const MgkGraphDesc& o, const MgkGraphDesc& i) {
        return (int64_t)o.nnz * (i.lane_len / 64) + 2 * (int64_t)o.n * (i.lane_len / 64);
    };
    const bool keep_atomic = b.max_deg > MGK_LANE_GROUP, swp_atomic = a.max_deg > MGK_LANE_GROUP;
    *swap = keep_atomic != swp_atomic ? keep_atomic : passes(b, a) < passes(a, b);
    const MgkGraphDesc& o = *swap ? b : a;
    const MgkGraphDesc& i = *swap ? a : b;
    MgkLargePair P{};
    P.g1 = *swap ? ib : ia;
    P.g2 = *swap ? ia : ib;
    P.n1 = o.n;
    P.n2 = i.n;
    const int64_t N = (int64_t)o.n * i.n;
    P.npad = (int32_t)((N + 63) & ~(int64_t)63);
    P.max_iter = max_iter_param > 0 ? max_iter_param : (int32_t)std::min<int64_t>(2 * N, 1000);
    P.nsteps = i.max_deg <= 1 ? 0 : i.max_deg <= 2 ? 1 : i.max_deg <= 4 ? 2 : i.max_deg <= 8 ? 3 : 4;
    P.atomic_rows = i.max_deg > MGK_LANE_GROUP ? 1 : 0;
    return P;
}

// Run Alg. 1 with global-memory vectors for a list of pairs (outer graphs from
// A, inner from B).  Synchronises the stream: the host watches the number of
// pairs still iterating.
mgk_status solve_large(mgk_ctx* ctx, const mgk_batch* A, const mgk_batch* Bb, int ia, int ib,
                       std::vector<MgkLargePair> pairs, bool dense, const MgkOutputs& out,
                       hipStream_t stream, const MgkParams& prm, bool weighted) {
    const int n_pairs = (int)pairs.size();
    if (n_pairs == 0) return MGK_OK;
    int64_t total = 0;
    int max_npad = 0, max_iter = 0, xmv_blocks = 1;
    int max_n1 = 1, max_n2 = 1, max_deg1 = 1, max_chunks = 1, min_chunks = 1 << 30;
    constexpr int CPB = MGK_LARGE_WAVES * MGK_LARGE_CHUNKS_PER_WAVE;
    for (MgkLargePair& P : pairs) {
        max_n1 = std::max(max_n1, P.n1);
        max_n2 = std::max(max_n2, P.n2);
        max_deg1 = std::max(max_deg1, A->graphs[P.g1].max_deg);
        max_chunks = std::max(max_chunks, Bb->graphs[P.g2].lane_len / 64);
        min_chunks = std::min(min_chunks, Bb->graphs[P.g2].lane_len / 64);
        P.vec = total;
        total += 5 * (int64_t)P.npad;
        max_npad = std::max(max_npad, P.npad);
        max_iter = std::max(max_iter, P.max_iter);
        const int chunks = Bb->graphs[P.g2].lane_len / 64;
        const int rb = (P.n1 + MGK_LARGE_ROWS_PER_BLOCK - 1) / MGK_LARGE_ROWS_PER_BLOCK;
        if (dense)
            xmv_blocks = std::max(xmv_blocks, (A->graphs[P.g1].n_tile_rows * Bb->graphs[P.g2].n_tile_rows + 3) / 4);
        else
            xmv_blocks = std::max(xmv_blocks, rb * ((chunks + CPB - 1) / CPB));
    }
    // Sparse product: stage the rows of p a row of the outer graph needs in LDS when a row
    // fits (one workgroup per outer row), else gather p from global memory.
    // Up to 60 KB of LDS per workgroup of at most 8 wavefronts (two or more workgroups per
    // CU); when the rows of p are so long that the neighbours of one outer row need more,
    // one workgroup of 16 wavefronts per CU with up to 120 KB.
    constexpr int kRowsLdsSmall = 60 * 1024, kRowsLdsLarge = 120 * 1024;
    int rows_threads = 0, rows_lds_bytes = 0, rows_chunks = 1;
    if (!dense && ctx->row_staging && (int64_t)max_n2 * 4 <= kRowsLdsLarge) {
        const int64_t need = (int64_t)max_deg1 * max_n2 * 4;
        const bool large = need > kRowsLdsSmall;
        const int budget = large ? kRowsLdsLarge : kRowsLdsSmall;
        const int rows = std::max(1, std::min(std::min(max_deg1, MGK_ROWS_MAX_BATCH), budget / (max_n2 * 4)));
        rows_lds_bytes = rows * max_n2 * 4;   // + the batch's outer entries and attributes, added by the launcher
        rows_threads = 64 * std::max(1, std::min(large ? 16 : 8, (max_chunks + 1) / 2));
        xmv_blocks = max_n1;
        // Chunks of the inner layout per pass of a wavefront: every outer entry read from LDS
        // then serves that many gathers.  Four need about 110 registers per lane, which only
        // the single large workgroup per CU affords; two where every wavefront still gets a
        // pass on the smallest pair.
        const int waves = rows_threads / 64;
        rows_chunks = large && min_chunks >= 4 * waves ? 4 : min_chunks >= 2 * waves ? 2 : 1;
    }
    const int vec_blocks = std::max(1, std::min(2048, (max_npad + 1023) / 1024));
    mgk_status st;
    if ((st = ensure(ctx, ctx->vec, (size_t)total * sizeof(float))) != MGK_OK) return st;
    if ((st = ensure(ctx, ctx->lpairs, (size_t)n_pairs * sizeof(MgkLargePair))) != MGK_OK) return st;
    if ((st = ensure(ctx, ctx->lstate, (size_t)n_pairs * sizeof(MgkPairState))) != MGK_OK) return st;
    if ((st = ensure(ctx, ctx->lactive, 64)) != MGK_OK) return st;
    if (!ctx->active_host) MGK_HIP(ctx, hipHostMalloc((void**)&ctx->active_host, 64, hipHostMallocDefault));

    // expanded entry lists of the batches involved (label scaling depends on the parameters)
    const mgk_batch* bt[2] = {A, Bb};
    const int slot[2] = {ia, ib};
    MgkExpanded ex[2] = {};
    MgkDenseTiles dt[2] = {};
    for (int k = 0; k < 2 && dense; ++k) {
        if (k == 1 && Bb == A) { dt[1] = dt[0]; break; }
        const size_t bytes = std::max<size_t>(16, (size_t)bt[k]->dev.n_tiles_total * 64 * sizeof(float));
        for (int a = 0; a < 3; ++a)
            if ((st = ensure(ctx, ctx->dense_tiles[slot[k]][a], bytes)) != MGK_OK) return st;
        float* dw = (float*)ctx->dense_tiles[slot[k]][0].p;
        float* de = (float*)ctx->dense_tiles[slot[k]][1].p;
        float* dlw = (float*)ctx->dense_tiles[slot[k]][2].p;
        hipError_t e = mgk_launch_expand_dense(bt[k]->dev, prm, dw, de, dlw, stream);
        if (e != hipSuccess) return fail(ctx, MGK_EDEVICE, "expand launch failed: %s", hipGetErrorString(e));
        dt[k].w = dw; dt[k].e = de; dt[k].lw = dlw;
    }
    for (int k = 0; k < 2 && !dense; ++k) {
        if (k == 1 && Bb == A) { ex[1] = ex[0]; break; }
        DevBuf& bo = ctx->exp_outer[slot[k]];
        DevBuf& bi = ctx->exp_inner[slot[k]];
        if ((st = ensure(ctx, bo, std::max<size_t>(16, (size_t)bt[k]->dev.nnz_total * sizeof(MgkEntry)))) != MGK_OK) return st;
        if ((st = ensure(ctx, bi, std::max<size_t>(16, (size_t)bt[k]->dev.lanes_total * sizeof(MgkEntry)))) != MGK_OK) return st;
        hipError_t e = mgk_launch_expand(bt[k]->dev, prm, (MgkEntry*)bo.p, (MgkEntry*)bi.p, stream);
        if (e != hipSuccess) return fail(ctx, MGK_EDEVICE, "expand launch failed: %s", hipGetErrorString(e));
        ex[k].outer = (const MgkEntry*)bo.p;
        ex[k].inner = (const MgkEntry*)bi.p;
    }

    MgkLargePair* dpairs = (MgkLargePair*)ctx->lpairs.p;
    MgkPairState* dstate = (MgkPairState*)ctx->lstate.p;
    int* dactive = (int*)ctx->lactive.p;
    float* vec = (float*)ctx->vec.p;
    // The pair records go through pinned memory owned by the context, so that the copy needs
    // no wait; the previous use of that buffer is waited for instead (long finished).
    {
        const size_t bytes = (size_t)n_pairs * sizeof(MgkLargePair);
        if (ctx->pin_busy) {
            MGK_HIP(ctx, hipEventSynchronize(ctx->pin_event));
            ctx->pin_busy = false;
        }
        if (bytes > ctx->pin_cap) {
            if (ctx->pin) MGK_HIP(ctx, hipHostFree(ctx->pin));
            ctx->pin = nullptr;
            ctx->pin_cap = 0;
            MGK_HIP(ctx, hipHostMalloc(&ctx->pin, bytes, hipHostMallocDefault));
            ctx->pin_cap = bytes;
        }
        if (!ctx->pin_event) MGK_HIP(ctx, hipEventCreateWithFlags(&ctx->pin_event, hipEventDisableTiming));
        memcpy(ctx->pin, pairs.data(), bytes);
        MGK_HIP(ctx, hipMemcpyAsync(dpairs, ctx->pin, bytes, hipMemcpyHostToDevice, stream));
    }
    MGK_HIP(ctx, hipMemsetAsync(dstate, 0, (size_t)n_pairs * sizeof(MgkPairState), stream));
    ctx->active_host[0] = n_pairs;   // pairs still iterating
    ctx->active_host[1] = 0;         // most iterations any pair needed
    MGK_HIP(ctx, hipMemcpyAsync(dactive, ctx->active_host, 2 * sizeof(int), hipMemcpyHostToDevice, stream));
    MGK_HIP(ctx, hipEventRecord(ctx->pin_event, stream));
    ctx->pin_busy = true;
    hipError_t e = mgk_launch_large_init(A->dev, Bb->dev, dpairs, dstate, vec, prm, n_pairs, vec_blocks, stream);
    if (e != hipSuccess) return fail(ctx, MGK_EDEVICE, "init launch failed: %s", hipGetErrorString(e));
    // The kernels of an iteration return at once for pairs that have stopped, so iterations
    // are enqueued without waiting: as many as the previous call of this kind needed, then
    // the host reads how many pairs still iterate, and goes on four at a time if any do.
    int it = 0;
    const int first_batch = std::max(1, std::min(max_iter, ctx->large_iter_guess));
    while (it < max_iter) {
        const int upto = it == 0 ? first_batch : std::min(max_iter, it + 4);
        for (; it < upto; ++it) {
            e = mgk_launch_large_iteration(A->dev, Bb->dev, ex[0], ex[1], dpairs, dstate, vec, prm, weighted,
                                           n_pairs, xmv_blocks, vec_blocks, dactive, it,
                                           dense ? &dt[0] : nullptr, dense ? &dt[1] : nullptr, rows_threads,
                                           rows_lds_bytes, rows_chunks, stream);
            if (e != hipSuccess) return fail(ctx, MGK_EDEVICE, "iteration launch failed: %s", hipGetErrorString(e));
        }
        MGK_HIP(ctx, hipMemcpyAsync(ctx->active_host, dactive, 2 * sizeof(int), hipMemcpyDeviceToHost, stream));
        MGK_HIP(ctx, hipStreamSynchronize(stream));
        ctx->pin_busy = false;
        if (ctx->active_host[0] <= 0) break;
    }
    if (ctx->active_host[0] <= 0) ctx->large_iter_guess = std::max(1, ctx->active_host[1]);
    log_launch(ctx, "%s pairs=%d iterations_enqueued=%d entries_cached=0 (+ mgk_large_dot / update / pupdate per iteration)",
               dense ? "mgk_large_xmv_dense_kernel" : rows_threads > 0 ? "mgk_large_xmv_rows_kernel" : "mgk_large_xmv_kernel",
               n_pairs, it);
    e = mgk_launch_large_final(A->dev, Bb->dev, ex[0], ex[1], dpairs, dstate, vec, prm, weighted, n_pairs, xmv_blocks,
                               vec_blocks, dense ? &dt[0] : nullptr, dense ? &dt[1] : nullptr, rows_threads,
                               rows_lds_bytes, rows_chunks, out, stream);
    if (e != hipSuccess) return fail(ctx, MGK_EDEVICE, "final launch failed: %s", hipGetErrorString(e));
    return MGK_OK;
}

mgk_status launch_jobs(mgk_ctx* ctx, const mgk_batch* X, const mgk_batch* Y, const JobList& jl,
                       const MgkOutputs& out, hipStream_t stream) {
    const MgkParams prm = make_params(ctx, X);
    const bool weighted = X->weighted || Y->weighted;
    ctx->launch_log.clear();
    for (const JobBin& b : jl.bins) {
        if (b.sell_regs > 0)
            log_launch(ctx, "mgk_pcg_sell<%d, %d, %d> pairs=%lld entries_cached=1", b.waves, b.ept, b.sell_regs, (long long)b.count);
        else if (b.chunks > 0)
            log_launch(ctx, "mgk_pcg_regs<%d, %d, %d, %d> pairs=%lld entries_cached=1", b.waves,
                       b.waves == 4 ? MGK_REGS_SMAX_W4 : MGK_REGS_SMAX_W8, b.ept, b.chunks, (long long)b.count);
        else
            log_launch(ctx, "mgk_pcg_small<%d, %d%s> pairs=%lld entries_cached=0", b.waves, b.ept,
                       b.atomic_rows ? ", atomic rows" : "", (long long)b.count);
        int64_t done = 0;
        while (done < b.count) {  // grid dimension limit
            const int64_t chunk = std::min<int64_t>(b.count - done, (int64_t)1 << 30);
            const MgkBatchDev& o = b.swapped ? Y->dev : X->dev;
            const MgkBatchDev& i = b.swapped ? X->dev : Y->dev;
            hipError_t e = b.sell_regs > 0
                ? mgk_launch_sell(b.waves, b.ept, b.sell_regs, o, i, jl.dev + b.first + done, (int)chunk, prm,
                                  b.lds_bytes, out, stream)
                : b.chunks > 0
                ? mgk_launch_regs(b.waves, b.chunks, b.ept, weighted, o, i, jl.dev + b.first + done, (int)chunk,
                                  prm, b.lds_bytes, out, stream)
                : mgk_launch_small(b.waves, b.ept, weighted, b.atomic_rows, o, i,
                                   jl.dev + b.first + done, (int)chunk, prm, b.lds_bytes, out, stream);
            if (e != hipSuccess)
                return fail(ctx, MGK_EDEVICE, "kernel launch failed: %s", hipGetErrorString(e));
            done += chunk;
        }
    }
    // Pairs with vectors in global memory go in groups: the pair index is a grid dimension
    // (at most 65535) and every pair of a group holds 5 vectors of scratch at the same time.
    constexpr size_t kMaxPairsPerGroup = 4096;
    constexpr int64_t kMaxScratchFloats = (int64_t)1 << 31;   // 8 GiB
    for (int dense = 0; dense < 2; ++dense)
        for (int swapped = 0; swapped < 2; ++swapped) {
            const std::vector<MgkLargePair>& all = jl.large[swapped][dense];
            size_t first = 0;
            while (first < all.size()) {
                size_t last = first;
                int64_t floats = 0;
                while (last < all.size() && last - first < kMaxPairsPerGroup &&
                       (last == first || floats + 5 * (int64_t)all[last].npad <= kMaxScratchFloats)) {
                    floats += 5 * (int64_t)all[last].npad;
                    ++last;
                }
                std::vector<MgkLargePair> group(all.begin() + (std::ptrdiff_t)first, all.begin() + (std::ptrdiff_t)last);
                const mgk_status st = swapped
                    ? solve_large(ctx, Y, X, 1, 0, std::move(group), dense != 0, out, stream, prm, weighted)
                    : solve_large(ctx, X, Y, 0, 1, std::move(group), dense != 0, out, stream, prm, weighted);
                if (st != MGK_OK) return st;
                first = last;
            }
        }
    return MGK_OK;
}

}  // namespace

// ============================================================================
extern "C" {

mgk_status mgk_create(mgk_ctx** out, int device) {
    if (!out) return MGK_EINVAL;
    *out = nullptr;
    if (device < -1) return MGK_EINVAL;
    if (device >= 0) {
        int count = 0;
        if (hipGetDeviceCount(&count) != hipSuccess || device >= count) return MGK_EDEVICE;
    }
    mgk_ctx* ctx = new (std::nothrow) mgk_ctx();
    if (!ctx) return MGK_ENOMEM;
    ctx->device = device;
    try { ctx->err.reserve(512); } catch (...) { delete ctx; return MGK_ENOMEM; }
    if (device >= 0 && hipSetDevice(device) != hipSuccess) { delete ctx; return MGK_EDEVICE; }
    *out = ctx;
    return MGK_OK;
}

void mgk_destroy(mgk_ctx* ctx) {
    if (!ctx) return;
    if (ctx->pair_jobs.dev) (void)hipFree(ctx->pair_jobs.dev);
    for (DevBuf* b : {&ctx->exp_outer[0], &ctx->exp_outer[1], &ctx->exp_inner[0], &ctx->exp_inner[1],
                      &ctx->vec, &ctx->lpairs, &ctx->lstate, &ctx->lactive, &ctx->nodal_off, &ctx->diag,
                      &ctx->dense_tiles[0][0], &ctx->dense_tiles[0][1], &ctx->dense_tiles[0][2],
                      &ctx->dense_tiles[1][0], &ctx->dense_tiles[1][1], &ctx->dense_tiles[1][2]})
        if (b->p) (void)hipFree(b->p);
    if (ctx->active_host) (void)hipHostFree(ctx->active_host);
    if (ctx->pin) (void)hipHostFree(ctx->pin);
    if (ctx->pin_event) (void)hipEventDestroy(ctx->pin_event);
    delete ctx;
}

const char* mgk_last_error(const mgk_ctx* ctx) { return ctx ? ctx->err.c_str() : "null context"; }

mgk_status mgk_set_vertex_kernel_delta(mgk_ctx* ctx, float h) {
    if (!ctx) return MGK_EINVAL;
    if (!(h > 0.f && h <= 1.f)) return fail(ctx, MGK_EINVAL, "vertex kernel h must be in (0, 1], got %g", h);
    ctx->h = h;
    return MGK_OK;
}

mgk_status mgk_set_edge_kernel_se(mgk_ctx* ctx, float length_scale) {
    if (!ctx) return MGK_EINVAL;
    if (!(length_scale > 0.f) || !std::isfinite(length_scale))
        return fail(ctx, MGK_EINVAL, "length scale must be positive and finite, got %g", length_scale);
    ctx->length_scale = length_scale;
    ctx->edge_kernel = MGK_EK_SE;
    ctx->label_dim = 1;
    return MGK_OK;
}

mgk_status mgk_set_edge_kernel_const(mgk_ctx* ctx, float c) {
    if (!ctx) return MGK_EINVAL;
    if (!(c >= 0.f && c <= 1.f)) return fail(ctx, MGK_EINVAL, "constant edge kernel must be in [0, 1], got %g", c);
    ctx->ke_const = c;
    ctx->edge_kernel = MGK_EK_CONST;
    ctx->label_dim = 1;
    return MGK_OK;
}

mgk_status mgk_set_edge_kernel_poly(mgk_ctx* ctx, int32_t n_coef, const float* coef, float rho) {
    if (!ctx) return MGK_EINVAL;
    if (n_coef < 1 || n_coef > MGK_POLY_MAX_COEF || !coef)
        return fail(ctx, MGK_EINVAL, "polynomial needs 1 to %d coefficients", MGK_POLY_MAX_COEF);
    if (!(rho > 0.f) || !std::isfinite(rho)) return fail(ctx, MGK_EINVAL, "support radius must be positive and finite, got %g", rho);
    for (int i = 0; i < n_coef; ++i)
        if (!std::isfinite(coef[i])) return fail(ctx, MGK_EINVAL, "coefficient %d is not finite", i);
    for (int k = 0; k <= 4096; ++k) {  // range of a base kernel (Section II-B)
        const double r = k / 4096.0;
        double v = 0.0;
        for (int i = n_coef - 1; i >= 0; --i) v = v * r + coef[i];
        if (v < -1e-6 || v > 1.0 + 1e-6)
            return fail(ctx, MGK_EINVAL, "polynomial is %g at r = %g, outside [0, 1]", v, r);
    }
    for (int i = 0; i < MGK_POLY_MAX_COEF; ++i) ctx->poly_c[i] = i < n_coef ? coef[i] : 0.f;
    ctx->poly_rho = rho;
    ctx->edge_kernel = MGK_EK_POLY;
    ctx->label_dim = 1;
    return MGK_OK;
}

static mgk_status set_attr_kernel(mgk_ctx* ctx, int kind, int32_t dim, const float* ls, int n_ls) {
    if (!ctx) return MGK_EINVAL;
    if (dim < 1 || dim > MGK_MAX_LABEL_DIM) return fail(ctx, MGK_EINVAL, "label attributes must be 1 to %d, got %d", MGK_MAX_LABEL_DIM, dim);
    if (!ls) return fail(ctx, MGK_EINVAL, "null length scales");
    for (int a = 0; a < n_ls; ++a)
        if (!(ls[a] > 0.f) || !std::isfinite(ls[a]))
            return fail(ctx, MGK_EINVAL, "length scale %d must be positive and finite, got %g", a, ls[a]);
    for (int a = 0; a < MGK_MAX_LABEL_DIM; ++a) ctx->attr_ls[a] = a < n_ls ? ls[a] : 1.f;
    ctx->edge_kernel = kind;
    ctx->label_dim = dim;
    return MGK_OK;
}

mgk_status mgk_set_edge_kernel_kron_se(mgk_ctx* ctx, int32_t dim, const float* length_scale) {
    return set_attr_kernel(ctx, MGK_EK_KRON_SE, dim, length_scale, dim);
}

mgk_status mgk_set_edge_kernel_rconv_se(mgk_ctx* ctx, int32_t dim, float length_scale) {
    return set_attr_kernel(ctx, MGK_EK_RCONV_SE, dim, &length_scale, 1);
}

mgk_status mgk_set_stop_prob(mgk_ctx* ctx, float q) {
    if (!ctx) return MGK_EINVAL;
    if (!(q > 0.f) || !std::isfinite(q)) return fail(ctx, MGK_EINVAL, "stopping probability must be > 0, got %g", q);
    ctx->q = q;
    return MGK_OK;
}

mgk_status mgk_set_solver(mgk_ctx* ctx, float rtol, int32_t max_iter) {
    if (!ctx) return MGK_EINVAL;
    if (!(rtol > 0.f) || !std::isfinite(rtol)) return fail(ctx, MGK_EINVAL, "rtol must be > 0, got %g", rtol);
    ctx->rtol = rtol;
    ctx->max_iter = max_iter;
    return MGK_OK;
}

mgk_status mgk_set_tile_path(mgk_ctx* ctx, int32_t mode) {
    if (!ctx) return MGK_EINVAL;
    if (mode < MGK_TILE_AUTO || mode > MGK_TILE_SPARSE_GATHER) return fail(ctx, MGK_EINVAL, "unknown tile path %d", mode);
    ctx->tile_path = mode;
    ctx->row_staging = mode == MGK_TILE_SPARSE_GATHER ? 0 : 1;
    return MGK_OK;
}

mgk_status mgk_set_onchip_limit(mgk_ctx* ctx, int32_t max_product) {
    if (!ctx) return MGK_EINVAL;
    if (max_product < 0) return fail(ctx, MGK_EINVAL, "on-chip limit must be >= 0, got %d", max_product);
    ctx->onchip_limit = std::min<int32_t>(max_product, MGK_SMALL_MAX_N);
    return MGK_OK;
}

mgk_status mgk_set_product_cache(mgk_ctx* ctx, int32_t enable) {
    if (!ctx) return MGK_EINVAL;
    if (enable < 0 || enable > 3) return fail(ctx, MGK_EINVAL, "product cache must be 0 to 3, got %d", enable);
    ctx->product_cache = enable;
    return MGK_OK;
}

mgk_status mgk_set_schedule(mgk_ctx* ctx, int32_t cost_sorted) {
    if (!ctx) return MGK_EINVAL;
    if (cost_sorted != 0 && cost_sorted != 1) return fail(ctx, MGK_EINVAL, "schedule must be 0 or 1, got %d", cost_sorted);
    ctx->cost_sorted = cost_sorted;
    return MGK_OK;
}

mgk_status mgk_set_launch(mgk_ctx* ctx, int32_t waves_per_pair) {
    if (!ctx) return MGK_EINVAL;
    const int w = waves_per_pair;
    if (!(w == 0 || w == 1 || w == 2 || w == 4 || w == 8 || w == 16))
        return fail(ctx, MGK_EINVAL, "waves_per_pair must be 0, 1, 2, 4, 8 or 16, got %d", w);
    ctx->waves = w;
    return MGK_OK;
}

// ----------------------------------------------------------------------------
mgk_status mgk_load_graphs(mgk_ctx* ctx, int32_t n_graphs, const int64_t* vtx_off,
                           const int32_t* vtx_label, const float* start_prob,
                           const int64_t* edge_off, const int32_t* src, const int32_t* dst,
                           const float* weight, const float* edge_label, int32_t reorder,
                           mgk_batch** out) {
    return mgk_load_graphs_attr(ctx, n_graphs, vtx_off, vtx_label, start_prob, edge_off, src, dst, weight,
                                1, edge_label, reorder, out);
}

static mgk_status load_graphs_body(mgk_ctx* ctx, int32_t n_graphs, const int64_t* vtx_off,
                                   const int32_t* vtx_label, const float* start_prob,
                                   const int64_t* edge_off, const int32_t* src, const int32_t* dst,
                                   const float* weight, int32_t label_dim, const float* edge_label,
                                   int32_t reorder, int32_t coord_dim, const float* coords, mgk_batch** out);

mgk_status mgk_load_graphs_attr(mgk_ctx* ctx, int32_t n_graphs, const int64_t* vtx_off,
                                const int32_t* vtx_label, const float* start_prob,
                                const int64_t* edge_off, const int32_t* src, const int32_t* dst,
                                const float* weight, int32_t label_dim, const float* edge_label,
                                int32_t reorder, mgk_batch** out) {
    return guarded(ctx, [&] {
        return load_graphs_body(ctx, n_graphs, vtx_off, vtx_label, start_prob, edge_off, src, dst, weight,
                                label_dim, edge_label, reorder, 0, nullptr, out);
    });
}

mgk_status mgk_load_graphs_embedded(mgk_ctx* ctx, int32_t n_graphs, const int64_t* vtx_off,
                                    const int32_t* vtx_label, const float* start_prob,
                                    const int64_t* edge_off, const int32_t* src, const int32_t* dst,
                                    const float* weight, const float* edge_label, int32_t coord_dim,
                                    const float* coords, mgk_batch** out) {
    return guarded(ctx, [&]() -> mgk_status {
        if (!ctx) return MGK_EINVAL;
        if (coord_dim < 1 || coord_dim > 3) return fail(ctx, MGK_EINVAL, "coordinates must have 1 to 3 dimensions, got %d", coord_dim);
        if (!coords) return fail(ctx, MGK_EINVAL, "coords is null");
        return load_graphs_body(ctx, n_graphs, vtx_off, vtx_label, start_prob, edge_off, src, dst, weight, 1,
                                edge_label, MGK_REORDER_MORTON, coord_dim, coords, out);
    });
}

static mgk_status load_graphs_body(mgk_ctx* ctx, int32_t n_graphs, const int64_t* vtx_off,
                                   const int32_t* vtx_label, const float* start_prob,
                                   const int64_t* edge_off, const int32_t* src, const int32_t* dst,
                                   const float* weight, int32_t label_dim, const float* edge_label,
                                   int32_t reorder, int32_t coord_dim, const float* coords, mgk_batch** out) {
    if (!ctx || !out) return MGK_EINVAL;
    *out = nullptr;
    if (label_dim < 1 || label_dim > MGK_MAX_LABEL_DIM)
        return fail(ctx, MGK_EINVAL, "label attributes must be 1 to %d, got %d", MGK_MAX_LABEL_DIM, label_dim);
    const int D = label_dim;
    if (n_graphs < 0 || !vtx_off || !edge_off) return fail(ctx, MGK_EINVAL, "null offsets or negative graph count");
    if (reorder < MGK_REORDER_NONE || reorder > MGK_REORDER_MORTON || (reorder == MGK_REORDER_MORTON && !coords))
        return fail(ctx, MGK_EINVAL, "unknown reorder mode %d (the space-filling-curve order needs mgk_load_graphs_embedded)", reorder);
    if (vtx_off[0] != 0 || edge_off[0] != 0) return fail(ctx, MGK_EINVAL, "offset arrays must start at 0");
    // every array below is sized by the last offsets: they must bound all the others
    for (int32_t g = 0; g < n_graphs; ++g) {
        if (vtx_off[g + 1] <= vtx_off[g]) return fail(ctx, MGK_EINVAL, "graph %d has no vertices", g);
        if (edge_off[g + 1] < edge_off[g]) return fail(ctx, MGK_EINVAL, "graph %d: edge offsets decrease", g);
    }
    const int64_t tot_v = vtx_off[n_graphs], tot_e = edge_off[n_graphs];
    if (tot_v > 0 && !vtx_label) return fail(ctx, MGK_EINVAL, "vtx_label is null");
    if (tot_e > 0 && (!src || !dst)) return fail(ctx, MGK_EINVAL, "src/dst is null");
    if (tot_v >= (int64_t)1 << 31 || 2 * tot_e >= (int64_t)1 << 31)
        return fail(ctx, MGK_ELIMIT, "batch too large for 32-bit offsets");

    mgk_batch* B = new (std::nothrow) mgk_batch();
    if (!B) return fail(ctx, MGK_ENOMEM, "out of host memory");
    struct Guard {
        mgk_batch* b;
        ~Guard() { if (b) { if (b->blob) (void)hipFree(b->blob); delete b; } }
    } guard{B};

    B->owner = ctx;
    B->n_graphs = n_graphs;
    B->graphs.resize(n_graphs);
    B->vtx_off.assign(vtx_off, vtx_off + n_graphs + 1);
    B->perm.resize((size_t)tot_v);
    std::vector<int32_t> vlabel((size_t)tot_v), rowptr((size_t)tot_v), lanepos((size_t)tot_v), iperm((size_t)tot_v), trow_ptr, tile_graph;
    std::vector<MgkSellVertex> sell_vtx;            // records of the owner-computes solver
    std::vector<MgkSellNbr> sell_nbr;
    B->sell_desc.reserve((size_t)n_graphs);
    std::vector<MgkEntry> list_outer, list_inner;   // nonzero lists for the register-resident solver
    std::vector<int32_t> regs_split;                // its division of every graph's rows among wavefronts
    list_outer.reserve((size_t)(2 * tot_e));
    // label attributes in the order of the two lists, attribute-major; filled after the loop
    // (the plane stride is the batch total): (position, edge) pairs collected meanwhile
    std::vector<std::pair<int64_t, int64_t>> attr_pos_outer, attr_pos_inner;
    B->label_dim = D;
    int64_t lanes_total = 0;
    std::vector<float> rowsum((size_t)tot_v), start((size_t)tot_v);
    B->w.reserve((size_t)(2 * tot_e));
    B->e.reserve((size_t)(2 * tot_e));
    double label_sum = 0.0;

    struct Nz { uint64_t key; float w, e; int64_t edge; };
    std::vector<Nz> nz;
    MgkAdj adj;
    std::vector<int32_t> cursor;

    // The vertex orders are by far the most expensive part of loading and independent per
    // graph: they are computed first, on several threads, for every graph whose edge list is
    // sound.  The loop below validates each graph in full (so errors are reported as before,
    // for the first bad graph) and only then takes the order computed here.
    std::vector<std::vector<int32_t>> pre_perm((size_t)n_graphs);
    if ((reorder == MGK_REORDER_PBR || reorder == MGK_REORDER_RCM) && n_graphs >= 8) {
        const int T = (int)std::max(1u, std::min({std::thread::hardware_concurrency(), 16u, (unsigned)n_graphs / 4u}));
        auto order_worker = [&](int t) {
          try {   // a worker that runs out of memory stops; the loop below orders what it left
            MgkAdj a;
            std::vector<int32_t> cur;
            for (int32_t g = t; g < n_graphs; g += T) {
                const int64_t v0 = vtx_off[g], v1 = vtx_off[g + 1], e0 = edge_off[g], e1 = edge_off[g + 1];
                if (v1 <= v0 || e1 < e0 || v1 - v0 > 65535 * (int64_t)kTile) continue;
                const int n = (int)(v1 - v0);
                bool sound = true;
                a.n = n;
                a.ptr.assign(n + 1, 0);
                for (int64_t k = e0; k < e1 && sound; ++k) {
                    const int32_t sv = src[k], dv = dst[k];
                    if (sv < 0 || sv >= n || dv < 0 || dv >= n || sv == dv) { sound = false; break; }
                    a.ptr[sv + 1]++;
                    a.ptr[dv + 1]++;
                }
                if (!sound) continue;
                for (int i = 0; i < n; ++i) a.ptr[i + 1] += a.ptr[i];
                a.idx.assign((size_t)(2 * (e1 - e0)), 0);
                cur.assign(a.ptr.begin(), a.ptr.end() - 1);
                for (int64_t k = e0; k < e1; ++k) {
                    a.idx[cur[src[k]]++] = dst[k];
                    a.idx[cur[dst[k]]++] = src[k];
                }
                for (int i = 0; i < n; ++i) std::sort(a.idx.begin() + a.ptr[i], a.idx.begin() + a.ptr[i + 1]);
                pre_perm[(size_t)g] = reorder == MGK_REORDER_PBR ? mgk_order_pbr(a, kTile) : mgk_order_rcm(a);
            }
          } catch (...) {
          }
        };
        JoiningThreads pool;
        for (int t = 1; t < T; ++t) pool.t.emplace_back(order_worker, t);
        order_worker(0);
        pool.join();
    }

    for (int32_t g = 0; g < n_graphs; ++g) {
        const int64_t v0 = vtx_off[g], v1 = vtx_off[g + 1], e0 = edge_off[g], e1 = edge_off[g + 1];
        if (v1 <= v0) return fail(ctx, MGK_EINVAL, "graph %d has no vertices", g);
        if (e1 < e0) return fail(ctx, MGK_EINVAL, "graph %d: edge offsets decrease", g);
        const int64_t n64 = v1 - v0, m = e1 - e0;
        if (n64 > 65535 * (int64_t)kTile) return fail(ctx, MGK_ELIMIT, "graph %d has too many vertices", g);
        const int n = (int)n64;

        // ---- validate edges, build adjacency (both directions)
        adj.n = n;
        adj.ptr.assign(n + 1, 0);
        for (int64_t k = e0; k < e1; ++k) {
            const int32_t s = src[k], d = dst[k];
            if (s < 0 || s >= n || d < 0 || d >= n)
                return fail(ctx, MGK_EINVAL, "graph %d edge %lld: endpoint out of range", g, (long long)(k - e0));
            if (s == d) return fail(ctx, MGK_EINVAL, "graph %d edge %lld: self loop", g, (long long)(k - e0));
            const float wv = weight ? weight[k] : 1.f;
            if (!(wv > 0.f) || !std::isfinite(wv))
                return fail(ctx, MGK_EINVAL, "graph %d edge %lld: weight must be finite and > 0", g, (long long)(k - e0));
            for (int a = 0; edge_label && a < D; ++a)
                if (!std::isfinite(edge_label[k * D + a]))
                    return fail(ctx, MGK_EINVAL, "graph %d edge %lld: label is not finite", g, (long long)(k - e0));
            adj.ptr[s + 1]++;
            adj.ptr[d + 1]++;
        }
        for (int i = 0; i < n; ++i) adj.ptr[i + 1] += adj.ptr[i];
        adj.idx.assign((size_t)(2 * m), 0);
        cursor.assign(adj.ptr.begin(), adj.ptr.end() - 1);
        for (int64_t k = e0; k < e1; ++k) {
            adj.idx[cursor[src[k]]++] = dst[k];
            adj.idx[cursor[dst[k]]++] = src[k];
        }
        for (int i = 0; i < n; ++i) {  // duplicate edges
            std::sort(adj.idx.begin() + adj.ptr[i], adj.idx.begin() + adj.ptr[i + 1]);
            if (std::adjacent_find(adj.idx.begin() + adj.ptr[i], adj.idx.begin() + adj.ptr[i + 1]) !=
                adj.idx.begin() + adj.ptr[i + 1])
                return fail(ctx, MGK_EINVAL, "graph %d: duplicate edge at vertex %d", g, i);
        }
        if (start_prob)
            for (int i = 0; i < n; ++i)
                if (!std::isfinite(start_prob[v0 + i]) || start_prob[v0 + i] < 0.f)
                    return fail(ctx, MGK_EINVAL, "graph %d vertex %d: bad starting probability", g, i);

        // ---- a2: vertex order
        std::vector<int32_t> perm;
        if (!pre_perm[(size_t)g].empty()) perm = std::move(pre_perm[(size_t)g]);
        else if (reorder == MGK_REORDER_PBR) perm = mgk_order_pbr(adj, kTile);
        else if (reorder == MGK_REORDER_RCM) perm = mgk_order_rcm(adj);
        else if (reorder == MGK_REORDER_MORTON) {
            for (int64_t k = v0 * coord_dim; k < v1 * coord_dim; ++k)
                if (!std::isfinite(coords[k])) return fail(ctx, MGK_EINVAL, "graph %d: coordinate is not finite", g);
            perm = mgk_order_morton(n, coord_dim, coords + v0 * coord_dim);
        } else perm = mgk_order_identity(n);
        std::copy(perm.begin(), perm.end(), B->perm.begin() + v0);

        // ---- per-vertex data in stored order; a1: row sums for d_i = sum_j A_ij + q
        std::vector<double> rs(n, 0.0);
        for (int64_t k = e0; k < e1; ++k) {
            const double wv = weight ? weight[k] : 1.0;
            rs[perm[src[k]]] += wv;
            rs[perm[dst[k]]] += wv;
        }
        for (int i = 0; i < n; ++i) {
            const int ni = perm[i];
            vlabel[v0 + ni] = vtx_label[v0 + i];
            iperm[v0 + ni] = i;
            start[v0 + ni] = start_prob ? start_prob[v0 + i] : 1.0f / (float)n;
            rowsum[v0 + ni] = (float)rs[ni];
        }

        // ---- a3: cut into octiles, drop empty ones, bitmap-pack
        const int ntr = (n + kTile - 1) / kTile;
        nz.clear();
        nz.reserve((size_t)(2 * m));
        for (int64_t k = e0; k < e1; ++k) {
            const float wv = weight ? weight[k] : 1.f;
            const float ev = edge_label ? edge_label[k * D] : 0.f;
            if (wv != 1.f) B->weighted = true;
            label_sum += 2.0 * ev;
            const int a = perm[src[k]], b = perm[dst[k]];
            for (int dir = 0; dir < 2; ++dir) {
                const int i = dir ? b : a, j = dir ? a : b;
                const uint64_t tile_id = (uint64_t)(i / kTile) * ntr + (uint64_t)(j / kTile);
                nz.push_back({tile_id * 64 + (uint64_t)((i % kTile) * 8 + (j % kTile)), wv, ev, k});
            }
        }
        std::sort(nz.begin(), nz.end(), [](const Nz& x, const Nz& y) { return x.key < y.key; });

        MgkGraphDesc& gd = B->graphs[g];
        gd.n = n;
        gd.nnz = (int32_t)nz.size();
        gd.n_tile_rows = ntr;
        gd.voff = (int32_t)v0;
        gd.zoff = (int32_t)B->w.size();
        gd.toff = (int32_t)B->tiles.size();
        gd.roff = (int32_t)trow_ptr.size();
        std::vector<int32_t> deg(n, 0);
        trow_ptr.resize(trow_ptr.size() + ntr + 1, 0);
        int32_t* trp = trow_ptr.data() + gd.roff;
        for (size_t k = 0; k < nz.size(); ++k) {
            const uint64_t tile_id = nz[k].key >> 6;
            const int bit = (int)(nz[k].key & 63);
            const int tr = (int)(tile_id / ntr), tc = (int)(tile_id % ntr);
            if (k == 0 || (nz[k - 1].key >> 6) != tile_id) {
                MgkTile t;
                t.tr = (uint16_t)tr;
                t.tc = (uint16_t)tc;
                t.nzoff = (uint32_t)k;
                t.bitmap = 0;
                B->tiles.push_back(t);
                trp[tr + 1]++;
                if (tr != tc) B->n_offdiag++;
            }
            B->tiles.back().bitmap |= 1ull << bit;
            B->w.push_back(nz[k].w);
            B->e.push_back(nz[k].e);
            deg[tr * kTile + bit / 8]++;
        }
        for (int r = 0; r < ntr; ++r) trp[r + 1] += trp[r];
        gd.n_tiles = (int32_t)B->tiles.size() - gd.toff;
        int32_t run = 0;
        for (int i = 0; i < n; ++i) { rowptr[v0 + i] = run; run += deg[i]; }
        // lane layout as inner operand: rows packed into groups of 16 lanes
        int32_t slot = 0, max_deg = 0;
        for (int i = 0; i < n; ++i) max_deg = std::max(max_deg, deg[i]);
        const bool packed = max_deg > MGK_LANE_GROUP;   // long rows: atomic adds anyway, no gaps
        for (int i = 0; i < n; ++i) {
            const int dg = deg[i];
            const int room = MGK_LANE_GROUP - slot % MGK_LANE_GROUP;
            if (!packed && dg > room && room != MGK_LANE_GROUP) slot += room;  // start a new group
            lanepos[v0 + i] = slot;
            slot += dg;
        }
        gd.max_deg = max_deg;
        gd.lane_len = (slot + 63) & ~63;
        gd.loff = (int32_t)lanes_total;
        {
            int32_t bounds[MGK_REGS_SPLIT_STRIDE];
            const int run4 = balanced_split(deg, n, 4, bounds);
            const int run8 = balanced_split(deg, n, 8, bounds + MGK_REGS_SPLIT_W8);
            regs_split.insert(regs_split.end(), bounds, bounds + MGK_REGS_SPLIT_STRIDE);
            gd.regs_runs = (int32_t)((uint32_t)std::min(run4, 0xffff) | ((uint32_t)std::min(run8, 0xffff) << 16));
        }
        lanes_total += gd.lane_len;
        if (lanes_total >= (int64_t)1 << 31) return fail(ctx, MGK_ELIMIT, "batch too large for 32-bit offsets");
        // the same nonzeros as plain lists: CSR order (columns ascending inside a row, which is
        // the order the octiles hold them in) and lane order
        list_outer.resize((size_t)gd.zoff + nz.size());
        list_inner.resize((size_t)gd.loff + gd.lane_len, MgkEntry{0u, 0u, 0u, 0u});
        std::vector<int32_t> filled(n, 0);
        for (size_t k = 0; k < nz.size(); ++k) {
            const uint64_t tile_id = nz[k].key >> 6;
            const int bit = (int)(nz[k].key & 63);
            const uint32_t i = (uint32_t)(tile_id / ntr) * kTile + bit / 8;
            const uint32_t j = (uint32_t)(tile_id % ntr) * kTile + bit % 8;
            const int rank = filled[i]++;
            uint32_t wbits, ebits;
            memcpy(&wbits, &nz[k].w, 4);
            memcpy(&ebits, &nz[k].e, 4);
            const bool row_end = rank + 1 == deg[i];
            list_outer[(size_t)gd.zoff + rowptr[v0 + i] + rank] =
                MgkEntry{i, j, ebits, wbits | (row_end ? 0x80000000u : 0u)};
            const MgkRunPos rp = mgk_run_pos(lanepos[v0 + i], rank, deg[i]);
            list_inner[(size_t)gd.loff + lanepos[v0 + i] + rank] =
                MgkEntry{i | (rp.rank << 20) | (rp.cut << 30) | (rp.last << 31), j, ebits, wbits};
            {
                attr_pos_outer.push_back({(int64_t)gd.zoff + rowptr[v0 + i] + rank, nz[k].edge});
                attr_pos_inner.push_back({(int64_t)gd.loff + lanepos[v0 + i] + rank, nz[k].edge});
            }
        }
        tile_graph.resize(B->tiles.size(), g);

        // ---- records of the owner-computes solver: vertices sorted by degree (descending),
        //      four neighbour records per vertex
        {
            MgkSellDesc sd{};
            sd.voff = (int32_t)sell_vtx.size();
            if (n <= MGK_SELL_MAX_N && max_deg <= MGK_SELL_MAX_DEG) {
                std::vector<int32_t> order(n), pos(n);
                std::iota(order.begin(), order.end(), 0);
                std::stable_sort(order.begin(), order.end(), [&](int32_t x, int32_t y) { return deg[x] > deg[y]; });
                for (int k = 0; k < n; ++k) pos[order[k]] = k;
                const int r8 = (n + 7) & ~7;
                for (int k = 0; k < r8; ++k) {
                    MgkSellVertex sv{0.f, 0.f, -1, 0xffffu};
                    MgkSellNbr sn[MGK_SELL_MAX_DEG] = {};   // weight 0, position 0: no entry
                    if (k < n) {
                        const int v = order[k];
                        sv.rowsum = rowsum[v0 + v];
                        sv.start = start[v0 + v];
                        sv.label = vlabel[v0 + v];
                        sv.id_deg = (uint32_t)v | ((uint32_t)deg[v] << 16);
                        for (int a = 0; a < deg[v]; ++a) {
                            const MgkEntry& en = list_outer[(size_t)gd.zoff + rowptr[v0 + v] + a];
                            const uint32_t wbits = en.w & 0x7fffffffu;
                            sn[a].pos = (uint32_t)pos[en.y];
                            memcpy(&sn[a].w, &wbits, 4);
                            memcpy(&sn[a].e, &en.z, 4);
                        }
                    }
                    sell_vtx.push_back(sv);
                    sell_nbr.insert(sell_nbr.end(), sn, sn + MGK_SELL_MAX_DEG);
                }
                uint32_t ga[MGK_SELL_MAX_DEG + 1] = {}, gb[MGK_SELL_MAX_DEG + 1] = {};
                for (int k = 0; k < n; k += MGK_SELL_OUTER_GROUP) ga[deg[order[k]]]++;
                for (int k = 0; k < n; k += MGK_SELL_INNER_GROUP) gb[deg[order[k]]]++;
                sd.ga03 = ga[0] | (ga[1] << 8) | (ga[2] << 16) | (ga[3] << 24);
                sd.gb03 = gb[0] | (gb[1] << 8) | (gb[2] << 16) | (gb[3] << 24);
                sd.hi = ga[4] | (gb[4] << 8) | (1u << 16);
            }
            B->sell_desc.push_back(sd);
        }
    }
    B->n_vertices = tot_v;
    B->nnz = (int64_t)B->w.size();
    B->n_tiles = (int64_t)B->tiles.size();
    B->label_mean = B->nnz ? label_sum / (double)B->nnz : 0.0;

    // ---- upload as one allocation
    std::vector<char> blob;
    const size_t o_g = append_bytes(blob, B->graphs);
    const size_t o_t = append_bytes(blob, B->tiles);
    const size_t o_w = append_bytes(blob, B->w);
    const size_t o_e = append_bytes(blob, B->e);
    const size_t o_vl = append_bytes(blob, vlabel);
    const size_t o_rs = append_bytes(blob, rowsum);
    const size_t o_st = append_bytes(blob, start);
    const size_t o_rp = append_bytes(blob, rowptr);
    const size_t o_lp = append_bytes(blob, lanepos);
    const size_t o_tr = append_bytes(blob, trow_ptr);
    const size_t o_tg = append_bytes(blob, tile_graph);
    const size_t o_ip = append_bytes(blob, iperm);
    const size_t o_lo = append_bytes(blob, list_outer);
    const size_t o_li = append_bytes(blob, list_inner);
    const size_t o_sp = append_bytes(blob, regs_split);
    std::vector<float> attr_outer, attr_inner;
    {
        attr_outer.assign((size_t)D * B->w.size(), 0.f);
        attr_inner.assign((size_t)D * (size_t)lanes_total, 0.f);
        for (const auto& pe : attr_pos_outer)
            for (int a = 0; a < D; ++a)
                attr_outer[(size_t)a * B->w.size() + (size_t)pe.first] = edge_label ? edge_label[pe.second * D + a] : 0.f;
        for (const auto& pe : attr_pos_inner)
            for (int a = 0; a < D; ++a)
                attr_inner[(size_t)a * (size_t)lanes_total + (size_t)pe.first] = edge_label ? edge_label[pe.second * D + a] : 0.f;
    }
    const size_t o_ao = append_bytes(blob, attr_outer);
    const size_t o_ai = append_bytes(blob, attr_inner);
    const size_t o_sd = append_bytes(blob, B->sell_desc);
    const size_t o_sv = append_bytes(blob, sell_vtx);
    const size_t o_sn = append_bytes(blob, sell_nbr);
    B->dev.label_dim = D;
    B->dev.uniform_start = start_prob ? 0 : 1;
    B->dev.n_graphs = n_graphs;
    B->dev.n_tiles_total = (int32_t)B->tiles.size();
    B->dev.nnz_total = (int32_t)B->w.size();
    B->dev.lanes_total = (int32_t)lanes_total;
    if (ctx->device < 0) {  // host-only context: packed form is kept for inspection only
        guard.b = nullptr;
        *out = B;
        return MGK_OK;
    }
    MGK_HIP(ctx, hipSetDevice(ctx->device));
    MGK_HIP(ctx, hipMalloc(&B->blob, blob.size()));
    MGK_HIP(ctx, hipMemcpy(B->blob, blob.data(), blob.size(), hipMemcpyHostToDevice));
    char* base = static_cast<char*>(B->blob);
    B->dev.graphs = reinterpret_cast<const MgkGraphDesc*>(base + o_g);
    B->dev.tiles = reinterpret_cast<const MgkTile*>(base + o_t);
    B->dev.w = reinterpret_cast<const float*>(base + o_w);
    B->dev.e = reinterpret_cast<const float*>(base + o_e);
    B->dev.vlabel = reinterpret_cast<const int32_t*>(base + o_vl);
    B->dev.rowsum = reinterpret_cast<const float*>(base + o_rs);
    B->dev.start = reinterpret_cast<const float*>(base + o_st);
    B->dev.rowptr = reinterpret_cast<const int32_t*>(base + o_rp);
    B->dev.lanepos = reinterpret_cast<const int32_t*>(base + o_lp);
    B->dev.trow_ptr = reinterpret_cast<const int32_t*>(base + o_tr);
    B->dev.tile_graph = reinterpret_cast<const int32_t*>(base + o_tg);
    B->dev.iperm = reinterpret_cast<const int32_t*>(base + o_ip);
    B->dev.list_outer = reinterpret_cast<const MgkEntry*>(base + o_lo);
    B->dev.list_inner = reinterpret_cast<const MgkEntry*>(base + o_li);
    B->dev.regs_split = reinterpret_cast<const int32_t*>(base + o_sp);
    B->dev.attr_outer = reinterpret_cast<const float*>(base + o_ao);
    B->dev.attr_inner = reinterpret_cast<const float*>(base + o_ai);
    B->dev.sell_desc = reinterpret_cast<const MgkSellDesc*>(base + o_sd);
    B->dev.sell_vtx = reinterpret_cast<const MgkSellVertex*>(base + o_sv);
    B->dev.sell_nbr = reinterpret_cast<const MgkSellNbr*>(base + o_sn);

    guard.b = nullptr;
    *out = B;
    return MGK_OK;
}

void mgk_free_batch(mgk_ctx* ctx, mgk_batch* batch) {
    if (!batch) return;
    (void)ctx;
    if (batch->blob || batch->gram_jobs.dev) (void)hipDeviceSynchronize();
    if (batch->gram_jobs.dev) (void)hipFree(batch->gram_jobs.dev);
    if (batch->blob) (void)hipFree(batch->blob);
    delete batch;
}

mgk_status mgk_batch_stats(const mgk_batch* b, int64_t* n_graphs, int64_t* n_vertices, int64_t* nnz,
                           int64_t* n_tiles, int64_t* n_offdiag_tiles) {
    if (!b) return MGK_EINVAL;
    if (n_graphs) *n_graphs = b->n_graphs;
    if (n_vertices) *n_vertices = b->n_vertices;
    if (nnz) *nnz = b->nnz;
    if (n_tiles) *n_tiles = b->n_tiles;
    if (n_offdiag_tiles) *n_offdiag_tiles = b->n_offdiag;
    return MGK_OK;
}

mgk_status mgk_batch_permutation(const mgk_batch* b, int32_t* perm_host) {
    if (!b || !perm_host) return MGK_EINVAL;
    std::copy(b->perm.begin(), b->perm.end(), perm_host);
    return MGK_OK;
}

mgk_status mgk_batch_get_tiles(const mgk_batch* b, int32_t g, int32_t* n_tiles, int32_t* nnz,
                               int32_t* tile_row, int32_t* tile_col, uint64_t* bitmap, float* w,
                               float* e) {
    if (!b || g < 0 || g >= b->n_graphs) return MGK_EINVAL;
    const MgkGraphDesc& gd = b->graphs[g];
    if (n_tiles) *n_tiles = gd.n_tiles;
    if (nnz) *nnz = gd.nnz;
    for (int t = 0; t < gd.n_tiles; ++t) {
        const MgkTile& tl = b->tiles[gd.toff + t];
        if (tile_row) tile_row[t] = tl.tr;
        if (tile_col) tile_col[t] = tl.tc;
        if (bitmap) bitmap[t] = tl.bitmap;
    }
    if (w) std::copy(b->w.begin() + gd.zoff, b->w.begin() + gd.zoff + gd.nnz, w);
    if (e) std::copy(b->e.begin() + gd.zoff, b->e.begin() + gd.zoff + gd.nnz, e);
    return MGK_OK;
}

// ----------------------------------------------------------------------------
static mgk_status gram_body(mgk_ctx* ctx, mgk_batch* batch, float* K_dev, int32_t* iters_dev,
                            int32_t* flag_dev, void* stream_);

mgk_status mgk_gram(mgk_ctx* ctx, mgk_batch* batch, float* K_dev, int32_t* iters_dev,
                    int32_t* flag_dev, void* stream_) {
    return guarded(ctx, [&] { return gram_body(ctx, batch, K_dev, iters_dev, flag_dev, stream_); });
}

static mgk_status gram_body(mgk_ctx* ctx, mgk_batch* batch, float* K_dev, int32_t* iters_dev,
                            int32_t* flag_dev, void* stream_) {
    if (!ctx || !batch || !K_dev) return fail(ctx, MGK_EINVAL, "null argument");
    if (batch->owner != ctx) return fail(ctx, MGK_ESTATE, "batch belongs to another context");
    if (ctx->device < 0) return fail(ctx, MGK_ESTATE, "host-only context cannot solve");
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    if (mgk_status st = check_label_dim(ctx, batch, batch)) return st;
    MGK_HIP(ctx, hipSetDevice(ctx->device));
    const int64_t G = batch->n_graphs;
    if (G * G >= (int64_t)1 << 31) return fail(ctx, MGK_ELIMIT, "Gram matrix too large for 32-bit output indices");
    if (batch->gram_jobs.dev != nullptr &&
        (batch->gram_jobs_waves != ctx->waves || batch->gram_jobs_max_iter != ctx->max_iter ||
         batch->gram_jobs_limit != ctx->onchip_limit || batch->gram_jobs_tile_path != ctx->tile_path ||
         batch->gram_jobs_cache != ctx->product_cache || batch->gram_jobs_sorted != ctx->cost_sorted ||
         batch->gram_jobs_attr_dim != attr_dim_of(ctx))) {
        MGK_HIP(ctx, hipStreamSynchronize(stream));  // launch shape changed: rebuild the job list
        MGK_HIP(ctx, hipFree(batch->gram_jobs.dev));
        batch->gram_jobs.dev = nullptr;
    }
    if (batch->gram_jobs.dev == nullptr && G > 0) {
        // a4: job list, one job per unordered pair, kept with the batch
        std::vector<HostJob> jobs;
        jobs.reserve((size_t)(G * (G + 1) / 2));
        for (auto& a : batch->gram_jobs.large) for (auto& v : a) v.clear();
        // the plans of the G (G + 1) / 2 pairs are independent: rows of the triangle in turn on
        // several threads, row i starting at pair i G - i (i - 1) / 2
        std::vector<PairPlan> plans((size_t)(G * (G + 1) / 2));
        {
            const int cache = ctx->product_cache;
            const int attr_dim = attr_dim_of(ctx);
            const int forced = ctx->waves, limit = ctx->onchip_limit;
            const int T = (int)std::max<int64_t>(1, std::min<int64_t>({(int64_t)std::thread::hardware_concurrency(), 16, G / 64}));
            auto plan_worker = [&](int t) {   // allocates nothing, cannot throw
                for (int64_t i = t; i < G; i += T) {
                    PairPlan* row = plans.data() + (i * G - i * (i - 1) / 2);
                    for (int64_t j = i; j < G; ++j)
                        row[j - i] = plan_pair(batch->graphs[i], batch->graphs[j], &batch->sell_desc[(size_t)i],
                                               &batch->sell_desc[(size_t)j], true, forced, limit, cache, attr_dim);
                }
            };
            JoiningThreads pool;
            for (int t = 1; t < T; ++t) pool.t.emplace_back(plan_worker, t);
            plan_worker(0);
            pool.join();
        }
        size_t next_plan = 0;
        for (int64_t i = 0; i < G; ++i)
            for (int64_t j = i; j < G; ++j) {
                const PairPlan pl = plans[next_plan++];
                HostJob hj;
                hj.job.g1 = (int32_t)(pl.swap ? j : i);
                hj.job.g2 = (int32_t)(pl.swap ? i : j);
                hj.job.out0 = (int32_t)(i * G + j);
                hj.job.out1 = i == j ? -1 : (int32_t)(j * G + i);
                hj.cost = pl.cost;
                hj.lds_words = (int32_t)pl.lds_words;
                hj.waves = (int16_t)pl.waves;
                hj.ept = (int16_t)pl.ept;
                hj.chunks = (int16_t)pl.chunks;
                hj.sell_regs = (int16_t)pl.sell_regs;
                hj.atomic_rows = pl.atomic_rows;
                hj.swapped = false;  // one batch: swapping is done through the indices
                if (pl.waves == 0) {  // vectors do not fit on chip
                    if ((int64_t)batch->graphs[i].n * batch->graphs[j].n >= ((int64_t)1 << 31) - 64)
                        return fail(ctx, MGK_ELIMIT, "pair (%lld, %lld) is too large", (long long)i, (long long)j);
                    bool sw;
                    MgkLargePair P = plan_large(batch->graphs[i], batch->graphs[j], (int32_t)i, (int32_t)j, &sw, ctx->max_iter);
                    P.out0 = hj.job.out0;
                    P.out1 = hj.job.out1;
                    batch->gram_jobs.large[0][use_dense_tiles(ctx, batch->graphs[i], batch->graphs[j]) ? 1 : 0].push_back(P);
                    continue;
                }
                jobs.push_back(hj);
            }
        mgk_status st = build_job_list(ctx, jobs, batch->gram_jobs, stream, nullptr);
        batch->gram_jobs_waves = ctx->waves;
        batch->gram_jobs_max_iter = ctx->max_iter;
        batch->gram_jobs_limit = ctx->onchip_limit;
        batch->gram_jobs_tile_path = ctx->tile_path;
        batch->gram_jobs_cache = ctx->product_cache;
        batch->gram_jobs_sorted = ctx->cost_sorted;
        batch->gram_jobs_attr_dim = attr_dim_of(ctx);
        if (st != MGK_OK) return st;
    }
    const MgkOutputs out{K_dev, iters_dev, flag_dev, nullptr, nullptr};
    return launch_jobs(ctx, batch, batch, batch->gram_jobs, out, stream);
}

// no_alloc: the job list goes to the fixed device array of mgk_noalloc.hip, pairs that need
// the global-memory solver (whose vectors the library would allocate) are refused, and no
// HIP allocation call is made on any path.
static mgk_status pairs_impl(mgk_ctx* ctx, mgk_batch* X, mgk_batch* Y, int64_t n_pairs,
                             const int32_t* i_host, const int32_t* j_host, float* K_dev,
                             float* x_dev, const int64_t* x_off_host, int32_t* iters_dev,
                             int32_t* flag_dev, void* stream_, bool no_alloc = false) {
    if (!ctx || !X || !Y) return fail(ctx, MGK_EINVAL, "null argument");
    if (X->owner != ctx || Y->owner != ctx) return fail(ctx, MGK_ESTATE, "batch belongs to another context");
    if (ctx->device < 0) return fail(ctx, MGK_ESTATE, "host-only context cannot solve");
    if (n_pairs < 0 || n_pairs >= (int64_t)1 << 31) return fail(ctx, MGK_EINVAL, "bad pair count");
    if (n_pairs == 0) return MGK_OK;
    if (!i_host || !j_host || !K_dev) return fail(ctx, MGK_EINVAL, "null argument");
    if (mgk_status st = check_label_dim(ctx, X, Y)) return st;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    MGK_HIP(ctx, hipSetDevice(ctx->device));
    // Either graph of a pair may be the outer operand; jobs whose outer graph
    // comes from Y are launched with the batch arguments exchanged.
    std::vector<HostJob> jobs((size_t)n_pairs);
    std::vector<MgkLargePair> large[2][2];
    for (int64_t k = 0; k < n_pairs; ++k) {
        const int32_t i = i_host[k], j = j_host[k];
        if (i < 0 || i >= X->n_graphs || j < 0 || j >= Y->n_graphs)
            return fail(ctx, MGK_EINVAL, "pair %lld: graph index out of range", (long long)k);
        const PairPlan pl = plan_pair(X->graphs[i], Y->graphs[j], &X->sell_desc[(size_t)i], &Y->sell_desc[(size_t)j], true,
                                      ctx->waves, ctx->onchip_limit, ctx->product_cache, attr_dim_of(ctx));
        HostJob& hj = jobs[(size_t)k];
        hj.job.g1 = pl.swap ? j : i;
        hj.job.g2 = pl.swap ? i : j;
        hj.job.out0 = (int32_t)k;
        hj.job.out1 = pl.swap ? MGK_OUT1_SWAPPED : MGK_OUT1_NONE;
        hj.cost = pl.cost;
        hj.lds_words = (int32_t)pl.lds_words;
        hj.waves = (int16_t)pl.waves;
        hj.ept = (int16_t)pl.ept;
        hj.chunks = (int16_t)pl.chunks;
        hj.sell_regs = (int16_t)pl.sell_regs;
        hj.atomic_rows = pl.atomic_rows;
        hj.swapped = pl.swap && X != Y;
        if (pl.waves == 0) {
            if (no_alloc)
                return fail(ctx, MGK_ELIMIT, "pair %lld (%d x %d vertices) needs the global-memory solver, "
                            "which allocates its vectors", (long long)k, X->graphs[i].n, Y->graphs[j].n);
            if ((int64_t)X->graphs[i].n * Y->graphs[j].n >= ((int64_t)1 << 31) - 64)
                return fail(ctx, MGK_ELIMIT, "pair %lld is too large", (long long)k);
            bool sw;
            MgkLargePair P = plan_large(X->graphs[i], Y->graphs[j], i, j, &sw, ctx->max_iter);
            P.out0 = (int32_t)k;
            P.out1 = sw ? MGK_OUT1_SWAPPED : MGK_OUT1_NONE;
            large[(sw && X != Y) ? 1 : 0][use_dense_tiles(ctx, X->graphs[i], Y->graphs[j]) ? 1 : 0].push_back(P);
            hj.waves = 0;
        }
    }
    if (ctx->pair_jobs_busy) {  // the previous call's kernels may still read the job buffer
        MGK_HIP(ctx, hipStreamSynchronize(ctx->pair_jobs_stream));
        ctx->pair_jobs_busy = false;
    }
    jobs.erase(std::remove_if(jobs.begin(), jobs.end(), [](const HostJob& h) { return h.waves == 0; }),
               jobs.end());
    MgkOutputs out{K_dev, iters_dev, flag_dev, nullptr, nullptr};
    if (no_alloc) {
        // Job list in the fixed array of this GPU.  All calls on the GPU share it: a call
        // that overlaps another one's kernels would overwrite the jobs they still read,
        // so within this context the previous such call is waited for first.
        if (ctx->fixed_jobs_busy) {
            MGK_HIP(ctx, hipStreamSynchronize(ctx->fixed_jobs_stream));
            ctx->fixed_jobs_busy = false;
        }
        JobList fixed;
        int64_t cap = 0;
        hipError_t e = mgk_noalloc_job_storage(ctx->device, &fixed.dev, &cap);
        if (e != hipSuccess) return fail(ctx, MGK_EDEVICE, "fixed job storage: %s", hipGetErrorString(e));
        mgk_status st = build_job_list(ctx, jobs, fixed, stream, &cap, true);
        if (st != MGK_OK) return st;
        ctx->fixed_jobs_stream = stream;
        ctx->fixed_jobs_busy = true;
        return launch_jobs(ctx, X, Y, fixed, out, stream);
    }
    mgk_status st = build_job_list(ctx, jobs, ctx->pair_jobs, stream, &ctx->pair_jobs_cap);
    if (st != MGK_OK) return st;
    for (int a = 0; a < 2; ++a)
        for (int b = 0; b < 2; ++b) ctx->pair_jobs.large[a][b] = std::move(large[a][b]);
    ctx->pair_jobs_stream = stream;
    ctx->pair_jobs_busy = true;
    if (x_dev) {
        if ((st = ensure(ctx, ctx->nodal_off, (size_t)n_pairs * sizeof(int64_t))) != MGK_OK) return st;
        MGK_HIP(ctx, hipMemcpyAsync(ctx->nodal_off.p, x_off_host, (size_t)n_pairs * sizeof(int64_t),
                                    hipMemcpyHostToDevice, stream));
        MGK_HIP(ctx, hipStreamSynchronize(stream));  // caller's array may be pageable
        out.nodal = x_dev;
        out.nodal_off = (const int64_t*)ctx->nodal_off.p;
    }
    return launch_jobs(ctx, X, Y, ctx->pair_jobs, out, stream);
}

mgk_status mgk_pairs(mgk_ctx* ctx, mgk_batch* X, mgk_batch* Y, int64_t n_pairs,
                     const int32_t* i_host, const int32_t* j_host, float* K_dev, int32_t* iters_dev,
                     int32_t* flag_dev, void* stream_) {
    return guarded(ctx, [&] {
        return pairs_impl(ctx, X, Y, n_pairs, i_host, j_host, K_dev, nullptr, nullptr, iters_dev, flag_dev, stream_);
    });
}

mgk_status mgk_pairs_dev(mgk_ctx* ctx, mgk_batch* X, mgk_batch* Y, int64_t n_pairs,
                         const int32_t* i_dev, const int32_t* j_dev, float* K_dev, int32_t* iters_dev,
                         int32_t* flag_dev, void* stream_) {
    return guarded(ctx, [&]() -> mgk_status {
        if (!ctx || !X || !Y) return fail(ctx, MGK_EINVAL, "null argument");
        if (ctx->device < 0) return fail(ctx, MGK_ESTATE, "host-only context cannot solve");
        if (n_pairs < 0 || n_pairs >= (int64_t)1 << 31) return fail(ctx, MGK_EINVAL, "bad pair count");
        if (n_pairs == 0) return MGK_OK;
        if (!i_dev || !j_dev) return fail(ctx, MGK_EINVAL, "null argument");
        // the launch shape of a pair is chosen on the host from the sizes of its graphs
        hipStream_t stream = static_cast<hipStream_t>(stream_);
        MGK_HIP(ctx, hipSetDevice(ctx->device));
        std::vector<int32_t> ij((size_t)(2 * n_pairs));
        MGK_HIP(ctx, hipMemcpyAsync(ij.data(), i_dev, (size_t)n_pairs * sizeof(int32_t), hipMemcpyDeviceToHost, stream));
        MGK_HIP(ctx, hipMemcpyAsync(ij.data() + n_pairs, j_dev, (size_t)n_pairs * sizeof(int32_t), hipMemcpyDeviceToHost, stream));
        MGK_HIP(ctx, hipStreamSynchronize(stream));
        return pairs_impl(ctx, X, Y, n_pairs, ij.data(), ij.data() + n_pairs, K_dev, nullptr, nullptr, iters_dev,
                          flag_dev, stream_);
    });
}

mgk_status mgk_pairs_noalloc(mgk_ctx* ctx, mgk_batch* X, mgk_batch* Y, int64_t n_pairs,
                             const int32_t* i_host, const int32_t* j_host, float* K_dev, int32_t* iters_dev,
                             int32_t* flag_dev, void* stream_) {
    return guarded(ctx, [&]() -> mgk_status {
        if (n_pairs > MGK_NOALLOC_MAX_PAIRS)
            return fail(ctx, MGK_ELIMIT, "mgk_pairs_noalloc takes at most %d pairs per call, got %lld",
                        MGK_NOALLOC_MAX_PAIRS, (long long)n_pairs);
        return pairs_impl(ctx, X, Y, n_pairs, i_host, j_host, K_dev, nullptr, nullptr, iters_dev, flag_dev, stream_,
                          true);
    });
}

mgk_status mgk_pairs_nodal(mgk_ctx* ctx, mgk_batch* X, mgk_batch* Y, int64_t n_pairs,
                           const int32_t* i_host, const int32_t* j_host, float* K_dev, float* x_dev,
                           const int64_t* x_off_host, int32_t* iters_dev, int32_t* flag_dev,
                           void* stream_) {
    if (n_pairs > 0 && (!x_dev || !x_off_host)) return fail(ctx, MGK_EINVAL, "null nodal output");
    return guarded(ctx, [&] {
        return pairs_impl(ctx, X, Y, n_pairs, i_host, j_host, K_dev, x_dev, x_off_host, iters_dev, flag_dev, stream_);
    });
}

int64_t mgk_launch_log(const mgk_ctx* ctx, char* buf, int64_t capacity) {
    if (!ctx) return -1;
    const int64_t need = (int64_t)ctx->launch_log.size() + 1;
    if (buf && capacity > 0) {
        const int64_t n = std::min<int64_t>(capacity - 1, (int64_t)ctx->launch_log.size());
        memcpy(buf, ctx->launch_log.data(), (size_t)n);
        buf[n] = 0;
    }
    return need;
}

mgk_status mgk_normalize_gram(mgk_ctx* ctx, int32_t n, float* K_dev, void* stream_) {
    if (!ctx || n < 0 || (n > 0 && !K_dev)) return fail(ctx, MGK_EINVAL, "bad argument");
    if (ctx->device < 0) return fail(ctx, MGK_ESTATE, "host-only context cannot solve");
    if (n == 0) return MGK_OK;
    MGK_HIP(ctx, hipSetDevice(ctx->device));
    mgk_status st = ensure(ctx, ctx->diag, (size_t)n * sizeof(float));
    if (st != MGK_OK) return st;
    hipError_t e = mgk_launch_normalize(K_dev, (float*)ctx->diag.p, n, static_cast<hipStream_t>(stream_));
    if (e != hipSuccess) return fail(ctx, MGK_EDEVICE, "normalize launch failed: %s", hipGetErrorString(e));
    return MGK_OK;
}

}  // extern "C"
