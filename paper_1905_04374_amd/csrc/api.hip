// C ABI of the multi-Bulyan library: argument checks, workspace layout, launch order.
// Every step of the rule runs in the kernels of dist.hip, select.hip, coordwise.hip and
// rowops.hip; nothing is computed on the host.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstring>
#include <map>
#include <mutex>
#include <vector>

#include "../../include/mbulyan.h"
#include "mb_internal.hpp"

namespace {

thread_local int tl_hip_error = 0;
int g_dist_algo = MB_DIST_AUTO;

int hip_fail(hipError_t e)
{
    tl_hip_error = (int)e;
    return MB_EHIP;
}
#define MB_HIP(expr)                                   \
    do {                                               \
        hipError_t e_ = (expr);                        \
        if (e_ != hipSuccess) return hip_fail(e_);     \
    } while (0)

// ---- workspace layout (offsets in bytes, every segment 256-byte aligned) ----
constexpr size_t kOffDist = 0;                                   // 64*64 doubles
constexpr size_t kOffReduced = kOffDist + 64 * 64 * 8;           // up to 2560 doubles
constexpr size_t kOffReduced2 = kOffReduced + 2560 * 8;          // the same of the second (centred) pass
constexpr size_t kOffGate = kOffReduced2 + 2560 * 8;             // flag and pivot row of the second pass
constexpr size_t kOffSel = kOffGate + 256;                       // 64 int32
constexpr size_t kOffM = kOffSel + 256;                          // 64 int32
constexpr size_t kOffSets = kOffM + 256;                         // 64*64 bytes
constexpr size_t kOffPlan = kOffSets + 4096;                     // plan of the Algorithm-1 coordinate pass
constexpr size_t kPlanBytes = 18 * 1024;
constexpr size_t kOffPrepIdx = kOffPlan + kPlanBytes;            // 2 x 64*64 bytes: neighbour by rank, rank by neighbour
constexpr size_t kOffPartials = kOffPrepIdx + 2 * 4096;
static_assert(mb::kPlanWords * sizeof(int32_t) <= kPlanBytes, "plan segment");
static_assert(MB_STORE_FP32 == mb::kStoreFp32 && MB_STORE_BF16 == mb::kStoreBf16 && MB_STORE_FP16 == mb::kStoreFp16,
              "the public storage codes are the kernels' own");

struct Workspace {
    char *base;
    size_t bytes;   // of the whole workspace: what follows kOffPartials holds the distance pass's partial sums
    // workgroups whose partial sums (stride doubles each) fit
    int max_blocks(int stride) const
    {
        const size_t room = bytes > kOffPartials ? (bytes - kOffPartials) / ((size_t)stride * sizeof(double)) : 0;
        return room > (size_t)mb::kGramMaxBlocks ? mb::kGramMaxBlocks : (int)room;
    }
    double *dist() const { return reinterpret_cast<double *>(base + kOffDist); }
    double *reduced() const { return reinterpret_cast<double *>(base + kOffReduced); }
    double *reduced2() const { return reinterpret_cast<double *>(base + kOffReduced2); }
    int *gate() const { return reinterpret_cast<int *>(base + kOffGate); }
    int32_t *sel() const { return reinterpret_cast<int32_t *>(base + kOffSel); }
    int32_t *m() const { return reinterpret_cast<int32_t *>(base + kOffM); }
    uint8_t *sets() const { return reinterpret_cast<uint8_t *>(base + kOffSets); }
    int32_t *plan() const { return reinterpret_cast<int32_t *>(base + kOffPlan); }
    // the rows of the distance matrix in ascending order, as the second distance pass leaves them for the
    // selection when a single matrix is aggregated (the matrix itself is then never written: same segment)
    double *prep_ordered() const { return dist(); }
    unsigned char *prep_idx() const { return reinterpret_cast<unsigned char *>(base + kOffPrepIdx); }
    double *partials() const { return reinterpret_cast<double *>(base + kOffPartials); }
};

int resolve_algo(int algo)
{
    if (algo == MB_DIST_AUTO) algo = g_dist_algo;
    if (algo == MB_DIST_AUTO) algo = MB_DIST_GRAM_BF16;   // fastest at every n measured (11..51)
    return algo;
}

size_t partial_bytes(int n, int64_t d)
{
    const int b1 = mb::dist_grid_blocks(d, MB_DIST_DIRECT), b2 = mb::dist_grid_blocks(d, MB_DIST_GRAM);
    const size_t s1 = (size_t)b1 * mb::kDirectSlots, s2 = (size_t)b2 * mb::gram_slots(n);
    return (s1 > s2 ? s1 : s2) * sizeof(double);
}

size_t workspace_bytes(int n, int64_t d)
{
    return kOffPartials + ((partial_bytes(n, d) + 255) / 256) * 256;
}

// ---- the library's own workspace, one per device --------------------------
struct Owned {
    void *ptr = nullptr;
    size_t bytes = 0;
};
std::mutex g_mu;
std::map<int, Owned> g_owned;

int own_workspace(size_t need, Workspace *ws)
{
    int dev = 0;
    MB_HIP(hipGetDevice(&dev));
    std::lock_guard<std::mutex> lock(g_mu);
    Owned &o = g_owned[dev];
    if (o.bytes < need) {
        if (o.ptr) {
            MB_HIP(hipDeviceSynchronize());
            MB_HIP(hipFree(o.ptr));
            o.ptr = nullptr;
            o.bytes = 0;
        }
        MB_HIP(hipMalloc(&o.ptr, need));
        o.bytes = need;
    }
    ws->base = static_cast<char *>(o.ptr);
    ws->bytes = o.bytes;
    return MB_OK;
}

int get_workspace(void *user, size_t user_bytes, int n, int64_t d, Workspace *ws)
{
    const size_t need = workspace_bytes(n, d);
    if (user) {
        if ((uintptr_t)user % 256 != 0 || user_bytes < need) return MB_EWORKSPACE;
        ws->base = static_cast<char *>(user);
        ws->bytes = user_bytes;
        return MB_OK;
    }
    return own_workspace(need, ws);
}

// ---- per-stage timing -------------------------------------------------------
struct Span {
    int stage;
    hipEvent_t a, b;
};
unsigned g_timing = 0;   // bit k: stage k is being timed
thread_local bool tl_no_timing = false;   // set while an entry point that must not create events runs
std::vector<Span> g_spans;
double g_ms[MB_NUM_STAGES] = {};
int64_t g_launches[MB_NUM_STAGES] = {};

struct StageTimer {
    bool on;
    Span sp;
    hipStream_t s;
    StageTimer(int stage, hipStream_t stream) : on(((g_timing >> stage) & 1u) && !tl_no_timing), s(stream)
    {
        if (!on) return;
        sp.stage = stage;
        if (hipEventCreate(&sp.a) != hipSuccess || hipEventCreate(&sp.b) != hipSuccess) { on = false; return; }
        (void)hipEventRecord(sp.a, s);
    }
    ~StageTimer()
    {
        if (!on) return;
        (void)hipEventRecord(sp.b, s);
        g_spans.push_back(sp);
    }
};

int drain_spans()
{
    for (Span &sp : g_spans) {
        float ms = 0.f;
        hipError_t e = hipEventSynchronize(sp.b);
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, sp.a, sp.b);
        (void)hipEventDestroy(sp.a);
        (void)hipEventDestroy(sp.b);
        if (e != hipSuccess) { g_spans.clear(); return hip_fail(e); }
        g_ms[sp.stage] += ms;
        g_launches[sp.stage] += 1;
    }
    g_spans.clear();
    return MB_OK;
}

// ---- argument checks ---------------------------------------------------------
int check_matrix(const void *grads, int n, int64_t d, int64_t ld)
{
    if (!grads || n < 1 || d < 1 || ld < d) return MB_EINVAL;
    if (n > MB_MAX_N) return MB_EUNSUPPORTED;
    return MB_OK;
}

// distances of one matrix into ws.dist()
// Gram form: first pass, its reduction, then the second (centred) pass, which finds out on the device
// whether it is needed (gram_combine.hpp) and returns at once if not.
// `defer` (may be null): leave the last step, Gram tiles -> distance matrix, to the selection kernel
// (it forms the matrix itself from ws.reduced(), ws.reduced2(), ws.gate()); set to 1 when that was possible.
// in16: mb::kStoreFp32, or gradients stored as 16-bit words (kStoreBf16 / kStoreFp16): Gram form only
// (one exact product per pair and coordinate)
int run_dist_gram(const void *grads, int in16, bool bf16, int n, int64_t d, int64_t ld, double *dist, int accumulate,
                  const Workspace &ws, hipStream_t s, int *defer)
{
    const int slots = mb::gram_slots(n);
    const int room = ws.max_blocks(slots);
    if (room < 1) return MB_EWORKSPACE;
    for (int pass = 0; pass < 2; ++pass) {
        // second pass: decides on the device whether it runs; its last workgroup reduces its tiles itself
        const double *first = pass ? ws.reduced() : nullptr;
        double *second_sums = pass ? ws.reduced2() : nullptr;
        int *gate = pass ? ws.gate() : nullptr;
        const bool prepare = pass && defer && !accumulate;   // the selection kernel will take it from here
        double *prep_ordered = prepare ? ws.prep_ordered() : nullptr;
        unsigned char *prep_idx = prepare ? ws.prep_idx() : nullptr;
        int nblocks = 0;
        {
            StageTimer t(pass ? MB_STAGE_REFINE : MB_STAGE_DIST, s);
            if (in16)
                MB_HIP(mb::launch_dist_gram_in16(static_cast<const uint16_t *>(grads), in16, n, d, ld, ws.partials(), room,
                                                 &nblocks, first, second_sums, gate, prep_ordered, prep_idx, s));
            else
                MB_HIP(mb::launch_dist_gram(static_cast<const float *>(grads), n, d, ld, ws.partials(), bf16, room,
                                            &nblocks, first, second_sums, gate, prep_ordered, prep_idx, s));
        }
        if (pass == 0) {
            StageTimer t(MB_STAGE_REDUCE, s);
            MB_HIP(mb::launch_reduce(ws.partials(), nblocks, slots, slots, ws.reduced(), ws.gate() + mb::kGateTicket, s));
        }
    }
    if (defer && !accumulate) {
        *defer = 1;
        return MB_OK;
    }
    StageTimer t(MB_STAGE_REDUCE, s);
    MB_HIP(mb::launch_finalize_gram(ws.reduced(), ws.reduced2(), ws.gate(), n, dist, accumulate, s));
    return MB_OK;
}

int run_dist_in16(const uint16_t *grads, int fmt, int n, int64_t d, int64_t ld, double *dist, int accumulate,
                  const Workspace &ws, hipStream_t s, int *defer = nullptr)
{
    return run_dist_gram(grads, fmt, true, n, d, ld, dist, accumulate, ws, s, defer);
}

int run_dist(const float *grads, int n, int64_t d, int64_t ld, double *dist, int accumulate, int algo,
             const Workspace &ws, hipStream_t s, int *defer = nullptr)
{
    algo = resolve_algo(algo);
    if (algo == MB_DIST_DIRECT) {
        int nblocks = mb::dist_grid_blocks(d, algo);
        const int nb = (n + 7) / 8, slots = nb * (nb + 1) / 2 * 64;
        const int room = ws.max_blocks(mb::kDirectSlots);
        if (room < 1) return MB_EWORKSPACE;
        nblocks = nblocks < room ? nblocks : room;
        {
            StageTimer t(MB_STAGE_DIST, s);
            MB_HIP(mb::launch_dist_direct(grads, n, d, ld, ws.partials(), nblocks, s));
        }
        StageTimer t(MB_STAGE_REDUCE, s);
        MB_HIP(mb::launch_reduce(ws.partials(), nblocks, mb::kDirectSlots, slots, ws.reduced(), nullptr, s));
        MB_HIP(mb::launch_finalize_direct(ws.reduced(), n, dist, accumulate, s));
        return MB_OK;
    }
    if (algo == MB_DIST_GRAM || algo == MB_DIST_GRAM_BF16)
        return run_dist_gram(grads, 0, algo == MB_DIST_GRAM_BF16, n, d, ld, dist, accumulate, ws, s, defer);
    return MB_EINVAL;
}

// plan_ready: the selection has already written the plan for (sel, sets)
int run_coord(const void *grads, int in16, int n, int64_t d, int64_t ld, int mode, int theta, int beta,
              const int32_t *sel, const uint8_t *sets, int32_t *plan, bool plan_ready, float *out, hipStream_t s)
{
    StageTimer t(MB_STAGE_COORD, s);
    if (mode == MB_MODE_SELECTED) {
        mb::CoordArgs a{grads, n, d, ld, sel, theta, beta, 0, out, in16};
        MB_HIP(mb::launch_coord_selected(a, s));
    } else {
        mb::CoordAlg1Args a{grads, n, d, ld, sel, sets, theta, beta, out, plan, in16};
        if (!plan_ready) MB_HIP(mb::launch_alg1_plan(n, theta, sel, sets, plan, s));
        MB_HIP(mb::launch_coord_alg1(a, s));
    }
    return MB_OK;
}

int resolve_params(int n, int f, int mode, int *theta, int *beta)
{
    int th = 0, be = 0;
    const int rc = mbulyan_params(n, f, mode, &th, &be);
    if (rc != MB_OK) return rc;
    if (*theta == 0) *theta = th;
    if (*beta == 0) *beta = (*theta == th) ? be : *theta - 2 * f;
    if (*theta < 1 || *theta > n || *beta < 1 || *beta > *theta) return MB_EINVAL;
    return MB_OK;
}

}  // namespace

namespace mb {
#define MB_BY_GROUP(PREFIX)                             \
    switch ((a.theta - 1) / 8) {                        \
        case 0: return PREFIX##0(a, s);                 \
        case 1: return PREFIX##1(a, s);                 \
        case 2: return PREFIX##2(a, s);                 \
        case 3: return PREFIX##3(a, s);                 \
        case 4: return PREFIX##4(a, s);                 \
        case 5: return PREFIX##5(a, s);                 \
        case 6: return PREFIX##6(a, s);                 \
        default: return PREFIX##7(a, s);                \
    }
hipError_t launch_coord_selected(const CoordArgs &a, hipStream_t s)
{
    if (a.theta < 1 || a.theta > kMaxN) return hipErrorInvalidValue;
    if (a.in16 == kStoreBf16) { MB_BY_GROUP(launch_coord16_group) }
    if (a.in16 == kStoreFp16) { MB_BY_GROUP(launch_coordh_group) }
    MB_BY_GROUP(launch_coord_group)
}
hipError_t launch_coord_alg1(const CoordAlg1Args &a, hipStream_t s)
{
    if (a.theta < 1 || a.theta > kMaxN) return hipErrorInvalidValue;
    if (a.in16 == kStoreBf16) { MB_BY_GROUP(launch_coord_alg1_16_group) }
    if (a.in16 == kStoreFp16) { MB_BY_GROUP(launch_coord_alg1_h_group) }
    MB_BY_GROUP(launch_coord_alg1_group)
}
#undef MB_BY_GROUP
}  // namespace mb

extern "C" {

const char *mbulyan_strerror(int status)
{
    switch (status) {
        case MB_OK: return "ok";
        case MB_EINVAL: return "invalid argument";
        case MB_EPRECOND: return "precondition violated: multi-Bulyan needs n >= 4f+3, multi-Krum n >= 2f+3";
        case MB_EUNSUPPORTED: return "unsupported size: n exceeds MB_MAX_N";
        case MB_EWORKSPACE: return "workspace too small or not 256-byte aligned";
        case MB_EHIP: return "HIP runtime error";
        default: return "unknown status";
    }
}

int mbulyan_last_hip_error(void) { return tl_hip_error; }

const char *mbulyan_version(void) { return "mbulyan 0.1 (gfx950)"; }

int mbulyan_params(int n, int f, int mode, int *theta, int *beta)
{
    if (n < 1 || f < 0 || (mode != MB_MODE_SELECTED && mode != MB_MODE_ALG1)) return MB_EINVAL;
    if (n < 4 * f + 3) return MB_EPRECOND;
    if (n > MB_MAX_N) return MB_EUNSUPPORTED;
    const int th = mode == MB_MODE_SELECTED ? n - 2 * f : n - 2 * f - 2;
    if (theta) *theta = th;
    if (beta) *beta = th - 2 * f;
    return MB_OK;
}

int mbulyan_workspace_bytes(int n, int64_t d, size_t *bytes)
{
    if (!bytes || n < 1 || d < 1) return MB_EINVAL;
    if (n > MB_MAX_N) return MB_EUNSUPPORTED;
    *bytes = workspace_bytes(n, d);
    return MB_OK;
}

int mbulyan_set_dist_algo(int algo)
{
    if (algo < MB_DIST_AUTO || algo > MB_DIST_GRAM_BF16) return MB_EINVAL;
    g_dist_algo = algo;
    return MB_OK;
}

int pairwise_sqdist(const float *grads, int n, int64_t d, int64_t ld, double *dist, int accumulate,
                    int algo, void *workspace, size_t ws_bytes, void *stream)
{
    int rc = check_matrix(grads, n, d, ld);
    if (rc != MB_OK) return rc;
    if (!dist) return MB_EINVAL;
    if (algo < MB_DIST_AUTO || algo > MB_DIST_GRAM_BF16) return MB_EINVAL;
    Workspace ws;
    rc = get_workspace(workspace, ws_bytes, n, d, &ws);
    if (rc != MB_OK) return rc;
    return run_dist(grads, n, d, ld, dist, accumulate ? 1 : 0, algo, ws, (hipStream_t)stream);
}

int krum_scores(const double *dist, int n, int f, const uint8_t *active, double *scores, void *stream)
{
    if (!dist || !scores || n < 1 || f < 0) return MB_EINVAL;
    if (n > MB_MAX_N) return MB_EUNSUPPORTED;
    StageTimer t(MB_STAGE_SELECT, (hipStream_t)stream);
    MB_HIP(mb::launch_select(dist, n, f, 1, active, nullptr, nullptr, nullptr, scores, nullptr, (hipStream_t)stream));
    return MB_OK;
}

int multikrum_select(const double *dist, int n, int f, int theta, int32_t *selected_idx,
                     uint8_t *agr_sets, int32_t *m_out, void *stream)
{
    if (!dist || !selected_idx || n < 1 || f < 0 || theta < 1 || theta > n) return MB_EINVAL;
    if (n > MB_MAX_N) return MB_EUNSUPPORTED;
    StageTimer t(MB_STAGE_SELECT, (hipStream_t)stream);
    MB_HIP(mb::launch_select(dist, n, f, theta, nullptr, selected_idx, agr_sets, m_out, nullptr, nullptr,
                             (hipStream_t)stream));
    return MB_OK;
}

int coordwise_trimmed_avg(const float *grads, int n, int64_t d, int64_t ld, const int32_t *selected_idx,
                          int theta, int beta, const uint8_t *agr_sets, float *out, void *stream)
{
    const int rc = check_matrix(grads, n, d, ld);
    if (rc != MB_OK) return rc;
    if (!selected_idx || !out || theta < 1 || theta > n || beta < 1 || beta > theta) return MB_EINVAL;
    Workspace ws{nullptr, 0};
    if (agr_sets) {   // the Algorithm-1 pass keeps its plan in the library's own workspace
        const int wrc = own_workspace(kOffPartials, &ws);
        if (wrc != MB_OK) return wrc;
    }
    return run_coord(grads, 0, n, d, ld, agr_sets ? MB_MODE_ALG1 : MB_MODE_SELECTED, theta, beta,
                     selected_idx, agr_sets, agr_sets ? ws.plan() : nullptr, false, out, (hipStream_t)stream);
}

static int aggregate_chunked(const void *const *chunks, int in16, int nchunks, const int64_t *chunk_d,
                             const int64_t *chunk_ld, int n, int f, int mode, float *const *outs,
                             int32_t *selected_idx, void *workspace, size_t ws_bytes, void *stream)
{
    if (!chunks || !chunk_d || !chunk_ld || !outs || nchunks < 1) return MB_EINVAL;
    int theta = 0, beta = 0;
    int rc = resolve_params(n, f, mode, &theta, &beta);
    if (rc != MB_OK) return rc;
    int64_t dmax = 0;
    for (int c = 0; c < nchunks; ++c) {
        rc = check_matrix(chunks[c], n, chunk_d[c], chunk_ld[c]);
        if (rc != MB_OK) return rc;
        if (!outs[c]) return MB_EINVAL;
        dmax = chunk_d[c] > dmax ? chunk_d[c] : dmax;
    }
    Workspace ws;
    rc = get_workspace(workspace, ws_bytes, n, dmax, &ws);
    if (rc != MB_OK) return rc;
    hipStream_t s = (hipStream_t)stream;
    for (int c = 0; c < nchunks; ++c) {
        rc = in16 ? run_dist_in16(static_cast<const uint16_t *>(chunks[c]), in16, n, chunk_d[c], chunk_ld[c], ws.dist(), c > 0,
                                  ws, s)
                  : run_dist(static_cast<const float *>(chunks[c]), n, chunk_d[c], chunk_ld[c], ws.dist(), c > 0,
                             MB_DIST_AUTO, ws, s);
        if (rc != MB_OK) return rc;
    }
    int32_t *sel = selected_idx ? selected_idx : ws.sel();   // the selection writes the caller's list in place
    {
        StageTimer t(MB_STAGE_SELECT, s);
        MB_HIP(mb::launch_select(ws.dist(), n, f, theta, nullptr, sel,
                                 mode == MB_MODE_ALG1 ? ws.sets() : nullptr, ws.m(), nullptr,
                                 mode == MB_MODE_ALG1 ? ws.plan() : nullptr, s));
    }
    for (int c = 0; c < nchunks; ++c) {
        rc = run_coord(chunks[c], in16, n, chunk_d[c], chunk_ld[c], mode, theta, beta, sel, ws.sets(), ws.plan(),
                       true, outs[c], s);
        if (rc != MB_OK) return rc;
    }
    return MB_OK;
}

int mbulyan_aggregate_chunked(const float *const *chunks, int nchunks, const int64_t *chunk_d,
                              const int64_t *chunk_ld, int n, int f, int mode, float *const *outs,
                              int32_t *selected_idx, void *workspace, size_t ws_bytes, void *stream)
{
    return aggregate_chunked(reinterpret_cast<const void *const *>(chunks), 0, nchunks, chunk_d, chunk_ld, n, f, mode,
                             outs, selected_idx, workspace, ws_bytes, stream);
}

int mbulyan_aggregate_chunked_bf16(const uint16_t *const *chunks, int nchunks, const int64_t *chunk_d,
                                   const int64_t *chunk_ld, int n, int f, int mode, float *const *outs,
                                   int32_t *selected_idx, void *workspace, size_t ws_bytes, void *stream)
{
    return aggregate_chunked(reinterpret_cast<const void *const *>(chunks), mb::kStoreBf16, nchunks, chunk_d, chunk_ld,
                             n, f, mode, outs, selected_idx, workspace, ws_bytes, stream);
}

int mbulyan_aggregate_chunked_fp16(const uint16_t *const *chunks, int nchunks, const int64_t *chunk_d,
                                   const int64_t *chunk_ld, int n, int f, int mode, float *const *outs,
                                   int32_t *selected_idx, void *workspace, size_t ws_bytes, void *stream)
{
    return aggregate_chunked(reinterpret_cast<const void *const *>(chunks), mb::kStoreFp16, nchunks, chunk_d, chunk_ld,
                             n, f, mode, outs, selected_idx, workspace, ws_bytes, stream);
}

// distance pass, reduction, selection, coordinate pass of one fp32 matrix on the workspace `ws`
static int aggregate_on(const Workspace &ws, const float *grads, int n, int f, int64_t d, int64_t ld, int mode,
                        int theta, int beta, float *out, int32_t *selected_idx, hipStream_t s)
{
    int deferred = 0;
    int rc = run_dist(grads, n, d, ld, ws.dist(), 0, MB_DIST_AUTO, ws, s, &deferred);
    if (rc != MB_OK) return rc;
    int32_t *sel = selected_idx ? selected_idx : ws.sel();   // the selection writes the caller's list in place
    {
        StageTimer t(MB_STAGE_SELECT, s);
        uint8_t *sets = mode == MB_MODE_ALG1 ? ws.sets() : nullptr;
        int32_t *plan = mode == MB_MODE_ALG1 ? ws.plan() : nullptr;   // written by the selection as well
        if (deferred)
            MB_HIP(mb::launch_select_gram(ws.reduced(), ws.reduced2(), ws.gate(), n, f, theta, sel, sets, ws.m(), plan,
                                          ws.prep_ordered(), ws.prep_idx(), s));
        else
            MB_HIP(mb::launch_select(ws.dist(), n, f, theta, nullptr, sel, sets, ws.m(), nullptr, plan, s));
    }
    return run_coord(grads, 0, n, d, ld, mode, theta, beta, sel, ws.sets(), ws.plan(), true, out, s);
}

int mbulyan_aggregate_ex(const float *grads, int n, int f, int64_t d, int64_t ld, int mode, int theta,
                         int beta, float *out, int32_t *selected_idx, void *workspace, size_t ws_bytes,
                         void *stream)
{
    int rc = check_matrix(grads, n, d, ld);
    if (rc != MB_OK) return rc;
    if (!out) return MB_EINVAL;
    rc = resolve_params(n, f, mode, &theta, &beta);
    if (rc != MB_OK) return rc;
    Workspace ws;
    rc = get_workspace(workspace, ws_bytes, n, d, &ws);
    if (rc != MB_OK) return rc;
    return aggregate_on(ws, grads, n, f, d, ld, mode, theta, beta, out, selected_idx, (hipStream_t)stream);
}

// ---- the same with nothing allocated: the workspace is a device array of the library itself ----
// Every device that loads the library holds its own copy of the array at its own address; the
// address is looked up once per device (with that device current) and used from then on.  The
// array's name in host code is only a handle for that lookup, never a pointer to pass on.
constexpr size_t kScratchBytes = (size_t)MB_NOALLOC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];
static_assert(kScratchBytes > kOffPartials + (size_t)mb::gram_slots(MB_MAX_N) * sizeof(double),
              "room for the fixed segments and at least one workgroup's partial sums");
constexpr int kMaxDevices = 64;
static void *g_scratch_ptr[kMaxDevices] = {};   // guarded by g_mu

static int scratch_workspace(Workspace *ws)
{
    int dev = 0;
    MB_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return hip_fail(hipErrorInvalidDevice);
    std::lock_guard<std::mutex> lock(g_mu);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        MB_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p || (uintptr_t)p % 256 != 0) return hip_fail(hipErrorInvalidSymbol);
        g_scratch_ptr[dev] = p;
    }
    ws->base = static_cast<char *>(g_scratch_ptr[dev]);
    ws->bytes = kScratchBytes;
    return MB_OK;
}

int mbulyan_aggregate_noalloc(const float *grads, int n, int f, int64_t d, int64_t ld, int mode, float *out,
                              int32_t *selected_idx, void *stream)
{
    int rc = check_matrix(grads, n, d, ld);   // n > MB_MAX_N: MB_EUNSUPPORTED, nothing is launched
    if (rc != MB_OK) return rc;
    if (!out) return MB_EINVAL;
    int theta = 0, beta = 0;
    rc = resolve_params(n, f, mode, &theta, &beta);
    if (rc != MB_OK) return rc;
    Workspace ws;
    rc = scratch_workspace(&ws);
    if (rc != MB_OK) return rc;
    if (ws.max_blocks(mb::gram_slots(n)) < 1) return MB_EWORKSPACE;
    // Nothing in the array has to start at zero: the distance pass overwrites the partial sums of
    // every workgroup it launches, and every later stage reads only what the stage before it wrote
    // in this call.  No timing events either (creating one may allocate).
    struct Quiet {
        Quiet() { tl_no_timing = true; }
        ~Quiet() { tl_no_timing = false; }
    } quiet;
    return aggregate_on(ws, grads, n, f, d, ld, mode, theta, beta, out, selected_idx, (hipStream_t)stream);
}

int mbulyan_aggregate(const float *grads, int n, int f, int64_t d, float *out, int32_t *selected_idx,
                      void *stream)
{
    return mbulyan_aggregate_ex(grads, n, f, d, d, MB_MODE_SELECTED, 0, 0, out, selected_idx, nullptr, 0,
                                stream);
}

int multikrum_aggregate(const float *grads, int n, int f, int64_t d, int64_t ld, float *out,
                        uint8_t *selected_mask, void *workspace, size_t ws_bytes, void *stream)
{
    int rc = check_matrix(grads, n, d, ld);
    if (rc != MB_OK) return rc;
    if (!out || f < 0) return MB_EINVAL;
    if (n < 2 * f + 3) return MB_EPRECOND;
    Workspace ws;
    rc = get_workspace(workspace, ws_bytes, n, d, &ws);
    if (rc != MB_OK) return rc;
    hipStream_t s = (hipStream_t)stream;
    int deferred = 0;
    rc = run_dist(grads, n, d, ld, ws.dist(), 0, MB_DIST_AUTO, ws, s, &deferred);
    if (rc != MB_OK) return rc;
    uint8_t *mask = selected_mask ? selected_mask : ws.sets();   // written in place by the selection
    {
        StageTimer t(MB_STAGE_SELECT, s);
        if (deferred)
            MB_HIP(mb::launch_select_gram(ws.reduced(), ws.reduced2(), ws.gate(), n, f, 1, ws.sel(), mask, ws.m(), nullptr,
                                          ws.prep_ordered(), ws.prep_idx(), s));
        else
            MB_HIP(mb::launch_select(ws.dist(), n, f, 1, nullptr, ws.sel(), mask, ws.m(), nullptr, nullptr, s));
    }
    {
        StageTimer t(MB_STAGE_COORD, s);
        MB_HIP(mb::launch_masked_mean(grads, n, d, ld, mask, out, s));
    }
    return MB_OK;
}

int coordwise_median(const float *grads, int n, int64_t d, int64_t ld, float *out, void *stream)
{
    const int rc = check_matrix(grads, n, d, ld);
    if (rc != MB_OK) return rc;
    if (!out) return MB_EINVAL;
    StageTimer t(MB_STAGE_COORD, (hipStream_t)stream);
    mb::CoordArgs a{grads, n, d, ld, nullptr, n, 1, 1, out, 0};
    MB_HIP(mb::launch_coord_selected(a, (hipStream_t)stream));
    return MB_OK;
}

// ---- gradients stored as 16-bit words (fmt = mb::kStoreBf16 / mb::kStoreFp16) ----------------
static int pairwise_sqdist_16(const uint16_t *grads, int fmt, int n, int64_t d, int64_t ld, double *dist,
                              int accumulate, void *workspace, size_t ws_bytes, void *stream)
{
    int rc = check_matrix(grads, n, d, ld);
    if (rc != MB_OK) return rc;
    if (!dist) return MB_EINVAL;
    Workspace ws;
    rc = get_workspace(workspace, ws_bytes, n, d, &ws);
    if (rc != MB_OK) return rc;
    return run_dist_in16(grads, fmt, n, d, ld, dist, accumulate ? 1 : 0, ws, (hipStream_t)stream);
}

static int coordwise_trimmed_avg_16(const uint16_t *grads, int fmt, int n, int64_t d, int64_t ld,
                                    const int32_t *selected_idx, int theta, int beta, const uint8_t *agr_sets,
                                    float *out, void *stream)
{
    const int rc = check_matrix(grads, n, d, ld);
    if (rc != MB_OK) return rc;
    if (!selected_idx || !out || theta < 1 || theta > n || beta < 1 || beta > theta) return MB_EINVAL;
    Workspace ws{nullptr, 0};
    if (agr_sets) {   // the Algorithm-1 pass keeps its plan in the library's own workspace
        const int wrc = own_workspace(kOffPartials, &ws);
        if (wrc != MB_OK) return wrc;
    }
    return run_coord(grads, fmt, n, d, ld, agr_sets ? MB_MODE_ALG1 : MB_MODE_SELECTED, theta, beta, selected_idx,
                     agr_sets, agr_sets ? ws.plan() : nullptr, false, out, (hipStream_t)stream);
}

static int multikrum_aggregate_16(const uint16_t *grads, int fmt, int n, int f, int64_t d, int64_t ld, float *out,
                                  uint8_t *selected_mask, void *workspace, size_t ws_bytes, void *stream)
{
    int rc = check_matrix(grads, n, d, ld);
    if (rc != MB_OK) return rc;
    if (!out || f < 0) return MB_EINVAL;
    if (n < 2 * f + 3) return MB_EPRECOND;
    Workspace ws;
    rc = get_workspace(workspace, ws_bytes, n, d, &ws);
    if (rc != MB_OK) return rc;
    hipStream_t s = (hipStream_t)stream;
    int deferred = 0;
    rc = run_dist_in16(grads, fmt, n, d, ld, ws.dist(), 0, ws, s, &deferred);
    if (rc != MB_OK) return rc;
    uint8_t *mask = selected_mask ? selected_mask : ws.sets();   // written in place by the selection
    {
        StageTimer t(MB_STAGE_SELECT, s);
        if (deferred)
            MB_HIP(mb::launch_select_gram(ws.reduced(), ws.reduced2(), ws.gate(), n, f, 1, ws.sel(), mask, ws.m(), nullptr,
                                          ws.prep_ordered(), ws.prep_idx(), s));
        else
            MB_HIP(mb::launch_select(ws.dist(), n, f, 1, nullptr, ws.sel(), mask, ws.m(), nullptr, nullptr, s));
    }
    {
        StageTimer t(MB_STAGE_COORD, s);
        MB_HIP(mb::launch_masked_mean_in16(grads, fmt, n, d, ld, mask, out, s));
    }
    return MB_OK;
}

static int coordwise_median_16(const uint16_t *grads, int fmt, int n, int64_t d, int64_t ld, float *out, void *stream)
{
    const int rc = check_matrix(grads, n, d, ld);
    if (rc != MB_OK) return rc;
    if (!out) return MB_EINVAL;
    StageTimer t(MB_STAGE_COORD, (hipStream_t)stream);
    mb::CoordArgs a{grads, n, d, ld, nullptr, n, 1, 1, out, fmt};
    MB_HIP(mb::launch_coord_selected(a, (hipStream_t)stream));
    return MB_OK;
}

static int mbulyan_aggregate_16(const uint16_t *grads, int fmt, int n, int f, int64_t d, int64_t ld, int mode,
                                int theta, int beta, float *out, int32_t *selected_idx, void *workspace,
                                size_t ws_bytes, void *stream)
{
    int rc = check_matrix(grads, n, d, ld);
    if (rc != MB_OK) return rc;
    if (!out || f < 0 || theta < 0 || beta < 0) return MB_EINVAL;
    if (mode != MB_MODE_SELECTED && mode != MB_MODE_ALG1) return MB_EINVAL;
    if (n < 4 * f + 3) return MB_EPRECOND;
    rc = resolve_params(n, f, mode, &theta, &beta);
    if (rc != MB_OK) return rc;
    Workspace ws;
    rc = get_workspace(workspace, ws_bytes, n, d, &ws);
    if (rc != MB_OK) return rc;
    hipStream_t s = (hipStream_t)stream;
    int deferred = 0;
    rc = run_dist_in16(grads, fmt, n, d, ld, ws.dist(), 0, ws, s, &deferred);
    if (rc != MB_OK) return rc;
    int32_t *sel = selected_idx ? selected_idx : ws.sel();   // the selection writes the caller's list in place
    {
        StageTimer t(MB_STAGE_SELECT, s);
        uint8_t *sets = mode == MB_MODE_ALG1 ? ws.sets() : nullptr;
        int32_t *plan = mode == MB_MODE_ALG1 ? ws.plan() : nullptr;   // written by the selection as well
        if (deferred)
            MB_HIP(mb::launch_select_gram(ws.reduced(), ws.reduced2(), ws.gate(), n, f, theta, sel, sets, ws.m(), plan,
                                          ws.prep_ordered(), ws.prep_idx(), s));
        else
            MB_HIP(mb::launch_select(ws.dist(), n, f, theta, nullptr, sel, sets, ws.m(), nullptr, plan, s));
    }
    return run_coord(grads, fmt, n, d, ld, mode, theta, beta, sel, ws.sets(), ws.plan(), true, out, s);
}

#define MB_16BIT_ENTRY_POINTS(SUFFIX, FMT)                                                                           \
    int pairwise_sqdist_##SUFFIX(const uint16_t *grads, int n, int64_t d, int64_t ld, double *dist, int accumulate,  \
                                 void *workspace, size_t ws_bytes, void *stream)                                     \
    {                                                                                                                \
        return pairwise_sqdist_16(grads, FMT, n, d, ld, dist, accumulate, workspace, ws_bytes, stream);              \
    }                                                                                                                \
    int coordwise_trimmed_avg_##SUFFIX(const uint16_t *grads, int n, int64_t d, int64_t ld,                          \
                                       const int32_t *selected_idx, int theta, int beta, const uint8_t *agr_sets,    \
                                       float *out, void *stream)                                                     \
    {                                                                                                                \
        return coordwise_trimmed_avg_16(grads, FMT, n, d, ld, selected_idx, theta, beta, agr_sets, out, stream);     \
    }                                                                                                                \
    int multikrum_aggregate_##SUFFIX(const uint16_t *grads, int n, int f, int64_t d, int64_t ld, float *out,         \
                                     uint8_t *selected_mask, void *workspace, size_t ws_bytes, void *stream)         \
    {                                                                                                                \
        return multikrum_aggregate_16(grads, FMT, n, f, d, ld, out, selected_mask, workspace, ws_bytes, stream);     \
    }                                                                                                                \
    int coordwise_median_##SUFFIX(const uint16_t *grads, int n, int64_t d, int64_t ld, float *out, void *stream)     \
    {                                                                                                                \
        return coordwise_median_16(grads, FMT, n, d, ld, out, stream);                                               \
    }                                                                                                                \
    int mbulyan_aggregate_##SUFFIX(const uint16_t *grads, int n, int f, int64_t d, int64_t ld, int mode, int theta,  \
                                   int beta, float *out, int32_t *selected_idx, void *workspace, size_t ws_bytes,    \
                                   void *stream)                                                                     \
    {                                                                                                                \
        return mbulyan_aggregate_16(grads, FMT, n, f, d, ld, mode, theta, beta, out, selected_idx, workspace,        \
                                    ws_bytes, stream);                                                               \
    }
MB_16BIT_ENTRY_POINTS(bf16, mb::kStoreBf16)
MB_16BIT_ENTRY_POINTS(fp16, mb::kStoreFp16)
#undef MB_16BIT_ENTRY_POINTS

int mbulyan_timing_enable(int stages)
{
    g_timing = static_cast<unsigned>(stages) & ((1u << MB_NUM_STAGES) - 1u);
    return MB_OK;
}

int mbulyan_timing_reset(void)
{
    const int rc = drain_spans();
    for (int i = 0; i < MB_NUM_STAGES; ++i) { g_ms[i] = 0; g_launches[i] = 0; }
    return rc;
}

int mbulyan_timing_read(double *ms_per_stage, int64_t *launches_per_stage)
{
    const int rc = drain_spans();
    if (rc != MB_OK) return rc;
    for (int i = 0; i < MB_NUM_STAGES; ++i) {
        if (ms_per_stage) ms_per_stage[i] = g_ms[i];
        if (launches_per_stage) launches_per_stage[i] = g_launches[i];
    }
    return MB_OK;
}

int mbulyan_release(void)
{
    drain_spans();
    std::lock_guard<std::mutex> lock(g_mu);
    int cur = 0;
    if (hipGetDevice(&cur) != hipSuccess) return hip_fail(hipGetLastError());
    for (auto &kv : g_owned) {
        if (!kv.second.ptr) continue;
        (void)hipSetDevice(kv.first);
        (void)hipDeviceSynchronize();
        (void)hipFree(kv.second.ptr);
        kv.second = Owned();
    }
    (void)hipSetDevice(cur);
    return MB_OK;
}

}  // extern "C"
