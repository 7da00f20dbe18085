// C ABI of the filtered int8 top-K library (see include/silvertorch.h for the contract).
// Host logic only: argument checks, filter grouping, scheduling, launches.  Every step of the
// hot path itself runs in the kernels of st_*_kernels.h.
#include "../../include/silvertorch.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <map>
#include <mutex>
#include <new>
#include <vector>

#include "st_stage_pool.h"
#include "st_bloom_kernels.h"
#include "st_mfma_kernels.h"
#include "st_ivf_kernels.h"
#include "st_quant_kernels.h"
#include "st_vm_kernels.h"
#include "st_plan.h"
#include "st_search_kernels.h"

// Workspace of st_search_static, the entry point for callers that may not allocate: device
// memory that exists from the moment the code object is loaded, one copy per GPU.
static __device__ __align__(256) unsigned char scratch[ST_STATIC_SCRATCH_BYTES];

namespace {

thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

// The C ABI never lets an exception out: host allocations that fail become ST_ENOMEM.
template <class F>
int guarded(F&& body)
{
    try {
        return body();
    } catch (const std::bad_alloc&) {
        return fail(ST_ENOMEM, "out of host memory");
    } catch (...) {
        return fail(ST_EINVAL, "unexpected failure in host code");
    }
}

#define ST_HIP(call)                                                                       \
    do {                                                                                   \
        hipError_t e_ = (call);                                                            \
        if (e_ != hipSuccess)                                                              \
            return fail(e_ == hipErrorOutOfMemory ? ST_ENOMEM : ST_EHIP,                   \
                        "%s failed: %s (%s:%d)", #call, hipGetErrorString(e_), __FILE__,   \
                        __LINE__);                                                         \
    } while (0)

// Test aid: the scorer a search of the calling thread is forced onto (0 auto, 1 wavefront dot
// product, 2 MFMA where it applies).  Per thread, so that one thread's setting never changes
// another thread's search.
thread_local int g_scoring_path = 0;

// Optional per-kernel timing with HIP events recorded on the caller's stream around each launch
// (state of the calling thread: the thread that begins a measurement makes the calls and ends it).
struct Timing {
    bool on = false;
    std::vector<hipEvent_t> ev;  // pairs: [2i] before, [2i+1] after launch i
    std::vector<int> kind;       // 0 scan, 1 select, 2 rescue, 3 filter expressions
    size_t used = 0;             // launches recorded
    size_t dropped = 0;
};
thread_local Timing g_timing;

struct TimedLaunch {
    hipStream_t stream;
    bool active;
    size_t slot;
    TimedLaunch(int kind, hipStream_t s) : stream(s), active(false), slot(0)
    {
        if (!g_timing.on) return;
        if (2 * (g_timing.used + 1) > g_timing.ev.size()) { ++g_timing.dropped; return; }
        slot = g_timing.used++;
        g_timing.kind[slot] = kind;
        active = hipEventRecord(g_timing.ev[2 * slot], stream) == hipSuccess;
    }
    ~TimedLaunch()
    {
        if (active) (void)hipEventRecord(g_timing.ev[2 * slot + 1], stream);
    }
};

// Pinned staging slots for the per-call tables (st_stage_pool.h): a call owns its slot from
// stage_get() until the StageHold goes out of scope, by which time the event behind the work that
// reads the slot has been recorded (or, on an error path after something was enqueued, the stream
// has been waited for).
st::StagePool g_pool;

bool stage_event_done(void* e)
{
    if (hipEventQuery((hipEvent_t)e) == hipSuccess) return true;
    (void)hipGetLastError();  // "not ready" must not show up as the next launch's error
    return false;
}

int stage_event_wait(void* e) { return hipEventSynchronize((hipEvent_t)e) == hipSuccess ? 0 : (int)ST_EHIP; }

struct StageHold {
    st::StageSlot* s = nullptr;
    hipStream_t stream = nullptr;
    bool enqueued = false;  // work that reads the slot is on the stream
    bool recorded = false;  // ... and the slot's event behind it
    void* host() const { return s->host; }
    void* dev_view() const { return s->dev_view; }
    ~StageHold()
    {
        if (!s) return;
        if (enqueued && !recorded) (void)hipStreamSynchronize(stream);
        g_pool.release(s, recorded);
    }
};

// Set while st_search_static runs in the calling thread: nothing may be allocated then.
thread_local bool t_no_alloc = false;

int stage_get(size_t bytes, hipStream_t stream, StageHold* h)
{
    st::StageSlot* s = nullptr;
    if (g_pool.acquire(stage_event_done, stage_event_wait, &s) != 0)
        return fail(ST_EHIP, "waiting for a staging slot failed");
    h->s = s;
    h->stream = stream;
    if (t_no_alloc && (!s->event || s->bytes < bytes))
        return fail(ST_EINVAL, "the tables of this batch (%zu bytes) exceed the pre-allocated staging slots (%zu bytes)",
                    bytes, s->bytes);
    if (!s->event) {
        hipEvent_t ev;
        ST_HIP(hipEventCreateWithFlags(&ev, hipEventDisableTiming));
        s->event = ev;
    }
    if (s->bytes < bytes) {  // owned and not pending: nothing reads the old memory any more
        if (s->host) ST_HIP(hipHostFree(s->host));
        s->host = nullptr;
        s->bytes = 0;
        const size_t want = std::max<size_t>(bytes, 64 * 1024);
        ST_HIP(hipHostMalloc(&s->host, want, hipHostMallocDefault));
        s->bytes = want;
        ST_HIP(hipHostGetDevicePointer(&s->dev_view, s->host, 0));
    }
    return ST_OK;
}

int stage_record(StageHold* h)
{
    ST_HIP(hipEventRecord((hipEvent_t)h->s->event, h->stream));
    h->recorded = true;
    return ST_OK;
}

// Per-device set-up, run by st_bloom_build (which allocates anyway and precedes every search on
// its device): the address of this device's copy of the static workspace, and, once per process,
// pinned memory and an event for every staging slot, so that st_search_static finds all of it in
// place.  In host code the array's name is only a handle for hipGetSymbolAddress; the address
// kept here is what kernels and copies are given.
constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices] = {};
std::mutex g_setup_mu;

int device_setup(int device)
{
    if (device < 0 || device >= kMaxDevices) return fail(ST_EINVAL, "device %d out of range", device);
    std::lock_guard<std::mutex> lock(g_setup_mu);
    if (!g_scratch_ptr[device]) {
        void* ptr = nullptr;
        ST_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        if (!ptr || ((uintptr_t)ptr & 255)) return fail(ST_EHIP, "static workspace has no usable device address");
        g_scratch_ptr[device] = ptr;
    }
    for (int i = 0; i < st::kStageSlots; ++i) {
        // slots nobody has used yet (a slot in use has its memory and event already)
        StageHold h;
        const int rc = stage_get(64 * 1024, nullptr, &h);
        if (rc != ST_OK) return rc;
    }
    return ST_OK;
}

bool is_device_pointer(const void* p)
{
    hipPointerAttribute_t attr;
    hipError_t e = hipPointerGetAttributes(&attr, p);
    if (e != hipSuccess) {
        (void)hipGetLastError();  // plain host memory reports an error: clear it
        return false;
    }
    return attr.type == hipMemoryTypeDevice || attr.type == hipMemoryTypeManaged;
}

// Distinct filters of a batch, as sorted lists of signature rows (Eq. 4: the bits QB sets).
// Groups are numbered in the order in which their first query appears; the queries of a group
// are listed in ascending order.
struct Groups {
    std::vector<int32_t> row_off, rows, q_off, q_list, q2grp;
    int32_t n_groups = 0;
};

// Per-thread buffers the host part of a search reuses from call to call, so that a call
// allocates nothing once the thread has seen the batch size.
struct GroupSet;
struct HostScratch;
HostScratch& host_scratch();

inline uint64_t hash_rows(const int32_t* r, int n)
{
    uint64_t h = 0xCBF29CE484222325ULL ^ (uint64_t)n;
    for (int i = 0; i < n; ++i) h = (h ^ (uint64_t)(uint32_t)r[i]) * 0x100000001B3ULL;
    return h ^ (h >> 29);
}

// Hashes every query's filter ids into signature rows, sorts and de-duplicates them, and groups
// the queries whose row lists are equal (open-addressing table over the lists' hashes).
int build_groups(const uint64_t* filt_ids, const int64_t* filt_off, int32_t n, int32_t m_bits,
                 int32_t k_hashes, Groups* out, std::vector<int32_t>& table, std::vector<int32_t>& tmp)
{
    constexpr int kMemoBits = 7;
    uint64_t memo_id[1 << kMemoBits];
    bool memo_ok[1 << kMemoBits] = {};
    int32_t memo_rows[1 << kMemoBits][ST_MAX_K_HASHES];
    int32_t cap = 16;
    while (cap < 2 * n) cap <<= 1;
    table.assign((size_t)cap, -1);
    out->q2grp.assign((size_t)n, 0);
    out->row_off.assign(1, 0);
    out->rows.clear();
    out->n_groups = 0;
    for (int32_t b = 0; b < n; ++b) {
        if (filt_off[b + 1] < filt_off[b]) return fail(ST_EINVAL, "filter offsets decrease at query %d", b);
        tmp.clear();
        for (int64_t a = filt_off[b]; a < filt_off[b + 1]; ++a) {
            // ids recur within a batch (few, broad filters): a small direct-mapped memo of this
            // call's hashes saves the 64-bit remainders
            const uint64_t id = filt_ids[a];
            const int slot = (int)((id * 0x9E3779B97F4A7C15ULL) >> (64 - kMemoBits));
            if (!memo_ok[slot] || memo_id[slot] != id) {
                for (int j = 0; j < k_hashes; ++j) memo_rows[slot][j] = (int32_t)st::bloom_bit(id, j, (uint32_t)m_bits);
                memo_id[slot] = id;
                memo_ok[slot] = true;
            }
            tmp.insert(tmp.end(), memo_rows[slot], memo_rows[slot] + k_hashes);
        }
        std::sort(tmp.begin(), tmp.end());
        const int32_t nr = (int32_t)(std::unique(tmp.begin(), tmp.end()) - tmp.begin());
        if (nr > ST_MAX_FILTER_BITS)
            return fail(ST_EINVAL, "filter of query %d sets %d signature bits (limit %d)", b, nr, ST_MAX_FILTER_BITS);
        int32_t g = -1;
        for (uint32_t at = (uint32_t)hash_rows(tmp.data(), nr) & (uint32_t)(cap - 1);; at = (at + 1) & (uint32_t)(cap - 1)) {
            const int32_t e = table[at];
            if (e < 0) {
                g = out->n_groups++;
                table[at] = g;
                out->rows.insert(out->rows.end(), tmp.begin(), tmp.begin() + nr);
                out->row_off.push_back((int32_t)out->rows.size());
                break;
            }
            const int32_t r0 = out->row_off[e], len = out->row_off[e + 1] - r0;
            if (len == nr && std::equal(tmp.begin(), tmp.begin() + nr, out->rows.begin() + r0)) {
                g = e;
                break;
            }
        }
        out->q2grp[b] = g;
    }
    // queries of each group, ascending (counting sort over the group numbers)
    out->q_off.assign((size_t)out->n_groups + 1, 0);
    for (int32_t b = 0; b < n; ++b) ++out->q_off[out->q2grp[b] + 1];
    for (int32_t g = 0; g < out->n_groups; ++g) out->q_off[g + 1] += out->q_off[g];
    out->q_list.assign((size_t)n, 0);
    tmp.assign(out->q_off.begin(), out->q_off.end() - 1);
    for (int32_t b = 0; b < n; ++b) out->q_list[tmp[out->q2grp[b]]++] = b;
    return ST_OK;
}

// One contiguous blob of int32 tables, each 16-byte aligned; uploaded in one copy.
struct Blob {
    std::vector<int32_t> data;
    size_t add(const std::vector<int32_t>& v)
    {
        const size_t at = data.size();
        data.insert(data.end(), v.begin(), v.end());
        data.resize((data.size() + 4) / 4 * 4, 0);  // pad (always leaves at least one spare int)
        return at * 4;
    }
    size_t bytes() const { return data.size() * 4; }
};

// A subset of the groups with its own tables (one per scorer).
struct GroupSet {
    std::vector<int32_t> row_off, rows, q_off, q_list;
    int32_t n = 0;
    void reset()
    {
        row_off.assign(1, 0);
        q_off.assign(1, 0);
        rows.clear();
        q_list.clear();
        n = 0;
    }
    void add(const Groups& all, int32_t g)
    {
        rows.insert(rows.end(), all.rows.begin() + all.row_off[g], all.rows.begin() + all.row_off[g + 1]);
        row_off.push_back((int32_t)rows.size());
        q_list.insert(q_list.end(), all.q_list.begin() + all.q_off[g], all.q_list.begin() + all.q_off[g + 1]);
        q_off.push_back((int32_t)q_list.size());
        ++n;
    }
};

struct SetAt { size_t row_off, rows, q_off, q_list; };

SetAt add_set(Blob& blob, const GroupSet& s)
{
    SetAt at;
    at.row_off = blob.add(s.row_off);
    at.rows = blob.add(s.rows);
    at.q_off = blob.add(s.q_off);
    at.q_list = blob.add(s.q_list);
    return at;
}

struct HostScratch {
    Groups groups;
    GroupSet set_mfma, set_dot;
    std::vector<int32_t> table, tmp, blk_off, blk_row, prow, q_taupos, q_prow;
    Blob blob;
};

HostScratch& host_scratch()
{
    thread_local HostScratch s;
    return s;
}

// Schedules depend on the sizes of a call only, and the planner tries several region capacities
// and segment sizes for each: results are kept (a few dozen shapes, oldest replaced first).
struct PlanKey {
    int64_t n_items;
    int32_t K, q_split, seg_cap, seed_ok, waves, min_cap, optimistic;
    bool operator==(const PlanKey& o) const
    {
        return n_items == o.n_items && K == o.K && q_split == o.q_split && seg_cap == o.seg_cap && seed_ok == o.seed_ok &&
               waves == o.waves && min_cap == o.min_cap && optimistic == o.optimistic;
    }
};
struct PlanEntry {
    PlanKey key;
    st::Plan plan;
    int rc;
    bool used = false;
};
constexpr int kPlanCache = 32;
PlanEntry g_plans[kPlanCache];
int g_plan_next = 0;
std::mutex g_plan_mu;

int cached_plan(int64_t n_items, int32_t K, int32_t q_split, int32_t seg_cap, int32_t batch_rows, st::Plan* out,
                int32_t waves = 2048, int32_t min_cap = 64, bool optimistic = true, bool small_first = false)
{
    // the batch enters the schedule only through "small enough for the seed pass"
    const PlanKey key{n_items, K, q_split, seg_cap, batch_rows <= st::kSeedMaxRows ? 1 : 0, waves, min_cap,
                      (optimistic ? 1 : 0) | (small_first ? 2 : 0)};
    {
        std::lock_guard<std::mutex> lock(g_plan_mu);
        for (const PlanEntry& e : g_plans)
            if (e.used && e.key == key) {
                if (e.rc == 0) *out = e.plan;
                return e.rc;
            }
    }
    st::Plan p;
    memset(&p, 0, sizeof(p));
    const int rc = st::make_plan(n_items, K, q_split, seg_cap, batch_rows, &p, waves, min_cap, optimistic, small_first);
    {
        std::lock_guard<std::mutex> lock(g_plan_mu);
        PlanEntry& e = g_plans[g_plan_next];
        g_plan_next = (g_plan_next + 1) % kPlanCache;
        e.key = key;
        e.plan = p;
        e.rc = rc;
        e.used = true;
    }
    if (rc == 0) *out = p;
    return rc;
}

// Likewise the configuration of the MFMA scan (split of the resident queries, wavefronts per
// workgroup, workgroups per compute unit), a function of four sizes.
struct MfmaCfgEntry {
    int32_t n_blocks, d, n_tasks, n_groups;
    int S, waves, wgs;
    bool used = false;
};
MfmaCfgEntry g_mfma_cfg[kPlanCache];
int g_mfma_cfg_next = 0;

void cached_mfma_config(int n_blocks, int d, int n_tasks, int n_groups, int* S, int* waves, int* wgs)
{
    {
        std::lock_guard<std::mutex> lock(g_plan_mu);
        for (const MfmaCfgEntry& e : g_mfma_cfg)
            if (e.used && e.n_blocks == n_blocks && e.d == d && e.n_tasks == n_tasks && e.n_groups == n_groups) {
                *S = e.S;
                *waves = e.waves;
                *wgs = e.wgs;
                return;
            }
    }
    st::mfma_choose_config(n_blocks, d, n_tasks, n_groups, 32, S, waves, wgs);
    std::lock_guard<std::mutex> lock(g_plan_mu);
    MfmaCfgEntry& e = g_mfma_cfg[g_mfma_cfg_next];
    g_mfma_cfg_next = (g_mfma_cfg_next + 1) % kPlanCache;
    e = MfmaCfgEntry{n_blocks, d, n_tasks, n_groups, *S, *waves, *wgs, true};
}

// Filter programs of a batch (Sec. 4.3: operation array run on a stack) as device tables for
// the expression kernel, and the queries grouped by distinct program.
struct ExprTables {
    std::vector<int32_t> prog_off{0}, code, leaf_rows;
    int32_t n_exprs = 0;
};

static_assert(ST_MAX_EXPR_OPS <= st::kExprOps && ST_MAX_EXPR_DEPTH <= st::kExprDepth &&
              ST_MAX_K_HASHES <= st::kExprHashes, "the expression kernel's LDS tables follow the limits");

// Stack discipline of one program: every operator finds its operands, one result is left
// (an empty program is the filter that passes everything), depth and length within the limits.
int check_program(const int32_t* ops, int64_t n, int32_t index)
{
    if (n > ST_MAX_EXPR_OPS) return fail(ST_EINVAL, "filter program %d has %lld entries (limit %d)", index, (long long)n, ST_MAX_EXPR_OPS);
    int depth = 0;
    for (int64_t i = 0; i < n; ++i) {
        switch (ops[i]) {
        case ST_OP_LEAF:
            if (++depth > ST_MAX_EXPR_DEPTH) return fail(ST_EINVAL, "filter program %d needs a stack deeper than %d", index, ST_MAX_EXPR_DEPTH);
            break;
        case ST_OP_AND:
        case ST_OP_OR:
            if (depth < 2) return fail(ST_EINVAL, "filter program %d: operator at entry %lld lacks operands", index, (long long)i);
            --depth;
            break;
        case ST_OP_NOT:
            if (depth < 1) return fail(ST_EINVAL, "filter program %d: NOT at entry %lld lacks an operand", index, (long long)i);
            break;
        default:
            return fail(ST_EINVAL, "filter program %d: unknown operation %d at entry %lld", index, ops[i], (long long)i);
        }
    }
    if (n > 0 && depth != 1) return fail(ST_EINVAL, "filter program %d leaves %d results", index, depth);
    return ST_OK;
}

// groups == nullptr: one expression per program, in order (mask export).  Otherwise equal
// programs share an expression, and group g tests row g of the evaluated masks.
int build_programs(const int32_t* ops, const uint64_t* ids, const int64_t* off, int32_t n, int32_t m_bits,
                   int32_t k_hashes, ExprTables* tab, Groups* groups)
{
    if (off[0] != 0) return fail(ST_EINVAL, "host_expr_offsets[0] must be 0");
    for (int32_t b = 0; b < n; ++b)
        if (off[b + 1] < off[b]) return fail(ST_EINVAL, "program offsets decrease at %d", b);
    if (off[n] > 0 && (!ops || !ids)) return fail(ST_EINVAL, "program arrays are null");
    std::map<std::pair<std::vector<int32_t>, std::vector<uint64_t>>, int32_t> index;
    std::vector<std::vector<int32_t>> members;
    if (groups) groups->q2grp.assign(n, 0);
    for (int32_t b = 0; b < n; ++b) {
        const int64_t len = off[b + 1] - off[b];
        const int rc = check_program(ops + off[b], len, b);
        if (rc != ST_OK) return rc;
        int32_t e = -1;
        if (groups) {
            std::vector<int32_t> o(ops + off[b], ops + off[b + 1]);
            std::vector<uint64_t> f(ids + off[b], ids + off[b + 1]);
            for (int64_t i = 0; i < len; ++i)
                if (o[i] != ST_OP_LEAF) f[i] = 0;  // ids of operators are not part of the program
            auto key = std::make_pair(std::move(o), std::move(f));
            auto it = index.find(key);
            if (it != index.end()) e = it->second;
            else index.emplace(std::move(key), tab->n_exprs);
        }
        if (e < 0) {
            e = tab->n_exprs++;
            for (int64_t i = off[b]; i < off[b + 1]; ++i) {
                tab->code.push_back(ops[i]);
                for (int j = 0; j < k_hashes; ++j)
                    tab->leaf_rows.push_back(ops[i] == ST_OP_LEAF ? (int32_t)st::bloom_bit(ids[i], j, (uint32_t)m_bits) : 0);
            }
            tab->prog_off.push_back((int32_t)tab->code.size());
            members.emplace_back();
        }
        members[e].push_back(b);
        if (groups) groups->q2grp[b] = e;
    }
    if (groups) {
        groups->n_groups = tab->n_exprs;
        groups->row_off.assign(1, 0);
        groups->q_off.assign(1, 0);
        groups->rows.clear();
        groups->q_list.clear();
        for (int32_t g = 0; g < tab->n_exprs; ++g) {
            groups->rows.push_back(g);
            groups->row_off.push_back(g + 1);
            groups->q_list.insert(groups->q_list.end(), members[g].begin(), members[g].end());
            groups->q_off.push_back((int32_t)groups->q_list.size());
        }
    }
    return ST_OK;
}

// Bytes of the device copy of the tables: offsets, then operators, then leaf rows.
size_t expr_table_bytes(int64_t n_programs, int64_t n_entries, int32_t k_hashes)
{
    return (size_t)st::round_up((n_programs + 1 + n_entries * (1 + (int64_t)k_hashes) + 4) * 4, 256);
}

}  // namespace

struct st_bloom {
    uint64_t* dev = nullptr;
    int64_t n_items = 0;
    int64_t n_tiles = 0;
    int32_t m_bits = 0;
    int32_t k_hashes = 0;
    int64_t bytes = 0;
    int device = 0;
};

extern "C" {

const char* st_last_error(void) { return g_err; }

int32_t st_version(void) { return 100; }

int32_t st_set_scoring_path(int32_t path)
{
    int32_t old = g_scoring_path;
    if (path >= 0 && path <= 2) g_scoring_path = path;
    return old;
}

int st_timing_begin(int32_t max_launches)
{
    return guarded([&]() -> int {
    if (max_launches < 1 || max_launches > (1 << 20)) return fail(ST_EINVAL, "max_launches out of range");
    while (g_timing.ev.size() < 2 * (size_t)max_launches) {
        hipEvent_t e;
        ST_HIP(hipEventCreate(&e));
        g_timing.ev.push_back(e);
    }
    g_timing.kind.assign(g_timing.ev.size() / 2, 0);
    g_timing.used = 0;
    g_timing.dropped = 0;
    g_timing.on = true;
    return ST_OK;
    });
}

int st_timing_end(double* out_ms, int64_t* out_launches)
{
    if (!out_ms || !out_launches) return fail(ST_EINVAL, "null argument");
    g_timing.on = false;
    for (int k = 0; k < 4; ++k) { out_ms[k] = 0.0; out_launches[k] = 0; }
    for (size_t i = 0; i < g_timing.used; ++i) {
        ST_HIP(hipEventSynchronize(g_timing.ev[2 * i + 1]));
        float ms = 0.f;
        ST_HIP(hipEventElapsedTime(&ms, g_timing.ev[2 * i], g_timing.ev[2 * i + 1]));
        out_ms[g_timing.kind[i]] += ms;
        out_launches[g_timing.kind[i]] += 1;
    }
    if (g_timing.dropped) return fail(ST_EINVAL, "%zu launches were not timed (raise max_launches)", g_timing.dropped);
    return ST_OK;
}

int64_t st_bloom_layout_bytes(int64_t n_items, int32_t m_bits)
{
    if (n_items < 0 || n_items >= (1LL << 31) || m_bits < 1 || m_bits > ST_MAX_M_BITS)
        return fail(ST_EINVAL, "bad sizes: n_items=%lld m_bits=%d", (long long)n_items, m_bits);
    const int64_t tiles = (n_items + st::kTileItems - 1) / st::kTileItems;
    return tiles * (int64_t)m_bits * st::kTileWords * 8;
}

int st_bloom_build(const int64_t* feat_offsets, const uint64_t* feat_ids, int64_t n_items,
                   int32_t m_bits, int32_t k_hashes, void* hip_stream, st_bloom** out)
{
    return guarded([&]() -> int {
    if (!out) return fail(ST_EINVAL, "out is null");
    *out = nullptr;
    if (!feat_offsets) return fail(ST_EINVAL, "feat_offsets is null");
    if (n_items < 0 || n_items >= (1LL << 31)) return fail(ST_EINVAL, "n_items=%lld out of range", (long long)n_items);
    if (m_bits < 1 || m_bits > ST_MAX_M_BITS) return fail(ST_EINVAL, "m_bits=%d out of range", m_bits);
    if (k_hashes < 1 || k_hashes > ST_MAX_K_HASHES) return fail(ST_EINVAL, "k_hashes=%d out of range", k_hashes);
    hipStream_t stream = (hipStream_t)hip_stream;

    st_bloom* b = new (std::nothrow) st_bloom;
    if (!b) return fail(ST_ENOMEM, "out of host memory");
    b->n_items = n_items;
    b->m_bits = m_bits;
    b->k_hashes = k_hashes;
    b->n_tiles = (n_items + st::kTileItems - 1) / st::kTileItems;
    b->bytes = st_bloom_layout_bytes(n_items, m_bits);
    int rc = ST_OK;
    int64_t* d_off = nullptr;
    uint64_t* d_ids = nullptr;
    auto body = [&]() -> int {
        ST_HIP(hipGetDevice(&b->device));
        const int rc_setup = device_setup(b->device);
        if (rc_setup != ST_OK) return rc_setup;
        if (b->bytes > 0) ST_HIP(hipMalloc((void**)&b->dev, (size_t)b->bytes));
        if (n_items == 0) return ST_OK;
        const int64_t* off = feat_offsets;
        const uint64_t* ids = feat_ids;
        int64_t nnz = 0;
        if (is_device_pointer(feat_offsets)) {
            ST_HIP(hipMemcpyAsync(&nnz, feat_offsets + n_items, 8, hipMemcpyDeviceToHost, stream));
            ST_HIP(hipStreamSynchronize(stream));
        } else {
            if (feat_offsets[0] != 0) return fail(ST_EINVAL, "feat_offsets[0] must be 0");
            for (int64_t i = 0; i < n_items; ++i)
                if (feat_offsets[i + 1] < feat_offsets[i]) return fail(ST_EINVAL, "feat_offsets decrease at item %lld", (long long)i);
            nnz = feat_offsets[n_items];
            ST_HIP(hipMalloc((void**)&d_off, (size_t)(n_items + 1) * 8));
            ST_HIP(hipMemcpyAsync(d_off, feat_offsets, (size_t)(n_items + 1) * 8, hipMemcpyHostToDevice, stream));
            off = d_off;
        }
        if (nnz < 0) return fail(ST_EINVAL, "negative feature count");
        if (nnz > 0 && !feat_ids) return fail(ST_EINVAL, "feat_ids is null");
        if (nnz > 0 && !is_device_pointer(feat_ids)) {
            ST_HIP(hipMalloc((void**)&d_ids, (size_t)nnz * 8));
            ST_HIP(hipMemcpyAsync(d_ids, feat_ids, (size_t)nnz * 8, hipMemcpyHostToDevice, stream));
            ids = d_ids;
        }
        const size_t lds = (size_t)std::min<int32_t>(m_bits, st::kBuildSlabRows) * st::kTileWords * 8;
        static std::atomic<bool> lds_set{false};
        if (!lds_set.load(std::memory_order_acquire)) {
            ST_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&st::bloom_build_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, st::kBuildSlabRows * st::kTileWords * 8));
            lds_set.store(true, std::memory_order_release);
        }
        {
            TimedLaunch t(0, stream);
            hipLaunchKernelGGL(st::bloom_build_kernel, dim3((unsigned)b->n_tiles), dim3(st::kBuildThreads), lds, stream, off,
                               ids, n_items, m_bits, k_hashes, b->dev);
        }
        ST_HIP(hipGetLastError());
        ST_HIP(hipStreamSynchronize(stream));
        return ST_OK;
    };
    rc = body();
    if (d_off) (void)hipFree(d_off);
    if (d_ids) (void)hipFree(d_ids);
    if (rc != ST_OK) {
        if (b->dev) (void)hipFree(b->dev);
        delete b;
        return rc;
    }
    *out = b;
    return ST_OK;
    });
}

int st_bloom_free(st_bloom* bloom)
{
    if (!bloom) return ST_OK;
    if (bloom->dev) ST_HIP(hipFree(bloom->dev));
    delete bloom;
    return ST_OK;
}

int64_t st_bloom_bytes(const st_bloom* bloom)
{
    if (!bloom) return fail(ST_EINVAL, "bloom is null");
    return bloom->bytes;
}

int64_t st_bloom_n_items(const st_bloom* bloom)
{
    if (!bloom) return fail(ST_EINVAL, "bloom is null");
    return bloom->n_items;
}

int st_bloom_export_signatures(const st_bloom* bloom, uint64_t* dev_out, void* hip_stream)
{
    if (!bloom || !dev_out) return fail(ST_EINVAL, "null argument");
    if (bloom->n_items == 0) return ST_OK;
    const unsigned grid = (unsigned)((bloom->n_items + 255) / 256);
    hipLaunchKernelGGL(st::bloom_export_kernel, dim3(grid), dim3(256), 0, (hipStream_t)hip_stream,
                       bloom->dev, bloom->n_items, bloom->m_bits, dev_out);
    ST_HIP(hipGetLastError());
    return ST_OK;
}

int st_bloom_mask(const st_bloom* bloom, const uint64_t* host_filt_ids, const int64_t* host_filt_offsets,
                  int32_t n_filters, uint64_t* dev_mask, void* hip_stream)
{
    return guarded([&]() -> int {
    if (!bloom || !host_filt_offsets || !dev_mask) return fail(ST_EINVAL, "null argument");
    if (n_filters < 0 || n_filters > 65535) return fail(ST_EINVAL, "n_filters=%d out of range", n_filters);
    if (host_filt_offsets[n_filters] > 0 && !host_filt_ids) return fail(ST_EINVAL, "host_filt_ids is null");
    if (n_filters == 0 || bloom->n_items == 0) return ST_OK;
    hipStream_t stream = (hipStream_t)hip_stream;
    // one row list per filter, in order (no grouping: the export is per filter)
    std::vector<int32_t> row_off(1, 0), rows;
    for (int32_t f = 0; f < n_filters; ++f) {
        if (host_filt_offsets[f + 1] < host_filt_offsets[f]) return fail(ST_EINVAL, "filter offsets decrease at %d", f);
        std::vector<int32_t> r;
        for (int64_t a = host_filt_offsets[f]; a < host_filt_offsets[f + 1]; ++a)
            for (int j = 0; j < bloom->k_hashes; ++j)
                r.push_back((int32_t)st::bloom_bit(host_filt_ids[a], j, (uint32_t)bloom->m_bits));
        std::sort(r.begin(), r.end());
        r.erase(std::unique(r.begin(), r.end()), r.end());
        rows.insert(rows.end(), r.begin(), r.end());
        row_off.push_back((int32_t)rows.size());
    }
    rows.push_back(0);
    int32_t* d_tab = nullptr;
    const size_t n_int = row_off.size() + rows.size();
    ST_HIP(hipMalloc((void**)&d_tab, n_int * 4));
    int rc = ST_OK;
    auto body = [&]() -> int {
        ST_HIP(hipMemcpyAsync(d_tab, row_off.data(), row_off.size() * 4, hipMemcpyHostToDevice, stream));
        ST_HIP(hipMemcpyAsync(d_tab + row_off.size(), rows.data(), rows.size() * 4, hipMemcpyHostToDevice, stream));
        const int64_t n_words = (bloom->n_items + 63) / 64;
        dim3 grid((unsigned)((n_words + 255) / 256), (unsigned)n_filters);
        hipLaunchKernelGGL(st::bloom_mask_kernel, grid, dim3(256), 0, stream, bloom->dev, bloom->m_bits,
                           bloom->n_items, n_words, d_tab, d_tab + row_off.size(), n_filters, dev_mask);
        ST_HIP(hipGetLastError());
        ST_HIP(hipStreamSynchronize(stream));
        return ST_OK;
    };
    rc = body();
    (void)hipFree(d_tab);
    return rc;
    });
}

int32_t st_search_plan(int64_t n_items, int32_t batch, int32_t K, int32_t q_split, int64_t* out_levels,
                       int32_t max_levels, int64_t* out_caps)
{
    if (n_items < 0 || n_items >= (1LL << 31) || batch < 1 || batch > ST_MAX_BATCH || K < 1 ||
        K > ST_MAX_TOP_K || q_split < 1 || q_split > 32 || (q_split & (q_split - 1)))
        return fail(ST_EINVAL, "bad sizes");
    st::Plan p;
    if (st::make_plan(n_items, K, q_split, st::kMaxSegItems, batch, &p) != 0)
        return fail(ST_EINVAL, "no schedule for these sizes");
    if (out_levels)
        for (int i = 0; i < p.n_levels && i < max_levels; ++i) {
            out_levels[3 * i + 0] = p.level[i].begin;
            out_levels[3 * i + 1] = p.level[i].end;
            out_levels[3 * i + 2] = (int64_t)p.level[i].seg_items * p.level[i].seg_per_visit;
        }
    if (out_caps) {
        out_caps[0] = p.groups;
        out_caps[1] = p.cap;
    }
    return p.n_levels;
}

static int64_t search_ws_bytes(int64_t n_items, int32_t d, int32_t batch, int32_t n_tasks, int32_t K, int32_t min_cap)
{
    if (n_items < 0 || n_items >= (1LL << 31)) return fail(ST_EINVAL, "n_items=%lld out of range", (long long)n_items);
    if (d < 16 || d > ST_MAX_DIM || d % 16) return fail(ST_EINVAL, "d=%d must be a multiple of 16 in [16, %d]", d, ST_MAX_DIM);
    if (batch < 1 || batch > ST_MAX_BATCH) return fail(ST_EINVAL, "batch=%d out of range", batch);
    if (n_tasks < 1 || n_tasks > ST_MAX_TASKS) return fail(ST_EINVAL, "n_tasks=%d out of range", n_tasks);
    if (K < 1 || K > ST_MAX_TOP_K) return fail(ST_EINVAL, "K=%d out of range", K);
    st::Plan p;
    if (cached_plan(n_items, K, 1, st::kMaxSegItems, batch * n_tasks, &p, 2048, min_cap) != 0)
        return fail(ST_EINVAL, "no schedule for these sizes");
    return (int64_t)st::make_layout(p, batch, K, d, n_tasks).total;
}

int64_t st_search_workspace_bytes(int64_t n_items, int32_t d, int32_t batch, int32_t n_tasks, int32_t K)
{
    return search_ws_bytes(n_items, d, batch, n_tasks, K, 64);
}

int64_t st_search_overflow_flags_offset(int64_t n_items, int32_t d, int32_t batch, int32_t n_tasks, int32_t K)
{
    const int64_t total = st_search_workspace_bytes(n_items, d, batch, n_tasks, K);
    if (total < 0) return total;
    st::Plan p;
    if (cached_plan(n_items, K, 1, st::kMaxSegItems, batch * n_tasks, &p) != 0)
        return fail(ST_EINVAL, "no schedule for these sizes");
    return (int64_t)st::make_layout(p, batch, K, d, n_tasks).ovf;
}

static int32_t plan_groups_per_row(int32_t q_split) { return st::scan_groups() / std::max(q_split, 1); }

static int search_impl(const st_bloom* bloom, const int8_t* dev_items, const float* dev_item_scale,
                       int64_t n_items, int32_t d, const int8_t* dev_queries, const float* dev_query_scale,
                       int32_t batch, int32_t n_tasks, const float* host_task_weight,
                       const uint64_t* host_filt_ids, const int64_t* host_filt_offsets, int32_t K,
                       int64_t* dev_out_ids, float* dev_out_scores, int32_t* dev_out_count,
                       void* dev_workspace, int64_t workspace_bytes, void* hip_stream,
                       const Groups* expr_groups = nullptr, const uint64_t* expr_rows = nullptr,
                       int32_t expr_row_count = 0, bool allow_seed = true, int32_t min_cap = 64,
                       int32_t* dry_out = nullptr)
{
    // dry_out: host part only (st_search_host_plan): no device pointer is looked at, nothing is
    // enqueued, and the summary of the schedule goes to dry_out[8]
    // allow_seed = false: no seed pass and no thresholds tighter than the K-th best so far (both
    // rest on a prefix of the corpus, which says nothing when the passing items sit in a few item
    // ranges, as after cluster probing)
    // expr_groups: the filters were evaluated beforehand into expr_row_count mask rows at
    // expr_rows, laid out like a Bloom index; each group then tests the one row it names
    if (!bloom) return fail(ST_EINVAL, "bloom is null");
    if (!host_filt_offsets && !expr_groups) return fail(ST_EINVAL, "null argument");
    if (!dry_out && (!dev_queries || !dev_query_scale || !dev_out_ids || !dev_out_scores || !dev_out_count || !dev_workspace))
        return fail(ST_EINVAL, "null argument");
    if (n_items != bloom->n_items)
        return fail(ST_EINVAL, "n_items=%lld but the index holds %lld", (long long)n_items, (long long)bloom->n_items);
    if (!dry_out && n_items > 0 && (!dev_items || !dev_item_scale)) return fail(ST_EINVAL, "null corpus");
    const int64_t need = search_ws_bytes(n_items, d, batch, n_tasks, K, min_cap);
    if (need < 0) return (int)need;
    if (!dry_out && workspace_bytes < need)
        return fail(ST_EWORKSPACE, "workspace has %lld bytes, %lld needed", (long long)workspace_bytes, (long long)need);
    if (((uintptr_t)dev_workspace & 255) || ((uintptr_t)dev_items & 15) || ((uintptr_t)dev_queries & 15) ||
        ((uintptr_t)dev_item_scale & 15))
        return fail(ST_EINVAL, "misaligned buffer (workspace 256 B; items, item scales and queries 16 B)");
    if (!expr_groups) {
        if (host_filt_offsets[0] != 0) return fail(ST_EINVAL, "host_filt_offsets[0] must be 0");
        if (host_filt_offsets[batch] > 0 && !host_filt_ids) return fail(ST_EINVAL, "host_filt_ids is null");
    }
    const bool weighted = host_task_weight != nullptr;
    if (weighted)
        for (int t = 0; t < n_tasks; ++t)
            if (!std::isfinite(host_task_weight[t])) return fail(ST_EINVAL, "task weight %d is not finite", t);
    hipStream_t stream = (hipStream_t)hip_stream;

    HostScratch& hs = host_scratch();
    Groups& groups = hs.groups;
    int rc = ST_OK;
    if (expr_groups)
        groups = *expr_groups;
    else
        rc = build_groups(host_filt_ids, host_filt_offsets, batch, bloom->m_bits, bloom->k_hashes, &groups, hs.table, hs.tmp);
    if (rc != ST_OK) return rc;

    // split the groups between the two scorers: MFMA where scoring is a real dense contraction
    // (enough query rows share the filter), the wavefront dot product otherwise
    const bool shape_ok = st::mfma_shape_ok(d, n_tasks) && g_scoring_path != 1;
    int min_rows = g_scoring_path == 2 ? 1 : st::kMfmaMinRows;
    if (shape_ok && min_rows > 1) {
        // a second scorer means a second pass over the corpus: when some group is dense enough
        // for MFMA, the small groups ride along unless their padding would more than double
        // the resident query blocks
        int64_t blocks_big = 0, blocks_all = 0;
        for (int32_t g = 0; g < groups.n_groups; ++g) {
            const int64_t rows = (int64_t)(groups.q_off[g + 1] - groups.q_off[g]) * n_tasks;
            blocks_all += (rows + 15) / 16;
            if (rows >= min_rows) blocks_big += (rows + 15) / 16;
        }
        if (blocks_big > 0 && blocks_all <= std::max<int64_t>(2 * blocks_big, blocks_big + 8)) min_rows = 1;
        // likewise, next to a dense group, when the padded rows of all groups together still fit four
        // rows of workgroups.  With no dense group at all (every query its own filter, single task)
        // the dot-product scorer takes the whole batch: 0.125 vs 0.152 ms of scan at 1M x 128, and
        // 0.093 vs 0.169 ms behind cluster probing, where most (query, segment) lists are empty.
        if (blocks_big > 0 && groups.n_groups <= st::kMfmaMaxGroups && blocks_all * 16 * d <= 4 * (int64_t)st::kMfmaQueryLds)
            min_rows = 1;
    }
    GroupSet &set_mfma = hs.set_mfma, &set_dot = hs.set_dot;
    set_mfma.reset();
    set_dot.reset();
    std::vector<int32_t>&blk_off = hs.blk_off, &blk_row = hs.blk_row;
    blk_off.assign(1, 0);
    blk_row.clear();
    for (int32_t g = 0; g < groups.n_groups; ++g) {
        const int32_t n_q = groups.q_off[g + 1] - groups.q_off[g];
        if (shape_ok && n_q * n_tasks >= min_rows && set_mfma.n < st::kMfmaMaxGroups) {
            set_mfma.add(groups, g);
            for (int32_t i = 0; i < n_q; ++i)
                for (int32_t t = 0; t < n_tasks; ++t) blk_row.push_back(groups.q_list[groups.q_off[g] + i] * n_tasks + t);
            blk_row.resize((blk_row.size() + 15) / 16 * 16, -1);
            blk_off.push_back((int32_t)(blk_row.size() / 16));
        } else {
            set_dot.add(groups, g);
        }
    }
    st::MfmaParams mp;
    memset(&mp, 0, sizeof(mp));
    mp.n_blocks = (int32_t)(blk_row.size() / 16);
    mp.q_split = 1;
    mp.waves = 4;
    mp.region_slots = 1;
    int mfma_wgs = 1;  // workgroups of the MFMA scan a compute unit holds at once
    if (set_mfma.n) {
        cached_mfma_config(mp.n_blocks, d, n_tasks, set_mfma.n, &mp.q_split, &mp.waves, &mfma_wgs);
        if (mp.q_split < 1) return fail(ST_EINVAL, "query batch too large for the resident-query scorer");
    }

    // 512-item segments fill the 16-item units better and halve the per-segment work, where the
    // larger per-wavefront lists leave as many workgroups on a compute unit
    mp.seg_stride = 256;
    if (set_mfma.n && st::mfma_lds_bytes(mp.n_blocks, mp.q_split, d, n_tasks, set_mfma.n, mp.waves,
                                         st::mfma_region_slots(mfma_wgs), st::kMfmaSegItems) * mfma_wgs <= 160 * 1024)
        mp.seg_stride = st::kMfmaSegItems;
    const int32_t seg_cap = set_mfma.n ? mp.seg_stride : st::kMaxSegItems;
    st::Plan plan;
    // wavefronts that scan a level side by side: the resident workgroups of one row of the grid
    const int32_t scan_waves = set_mfma.n ? std::max(1, std::min(plan_groups_per_row(mp.q_split), st::kComputeUnits * mfma_wgs / mp.q_split)) * mp.waves
                                          : st::scan_groups();  // (a whole workgroup shares a segment there)
    // (searches that will take their first level as a sample spread over the corpus -- the condition of
    // samp_stride below -- may plan a smaller one)
    const bool spread_first = allow_seed && set_mfma.n && !set_dot.n && mp.waves == 8;
    if (cached_plan(n_items, K, mp.q_split, seg_cap, allow_seed ? batch * n_tasks : st::kSeedMaxRows + 1, &plan, scan_waves,
                    min_cap, allow_seed, spread_first) != 0)
        return fail(ST_EINVAL, "no schedule for these sizes");
    st::Plan plan1;
    if (cached_plan(n_items, K, 1, st::kMaxSegItems, batch * n_tasks, &plan1, 2048, min_cap) != 0)
        return fail(ST_EINVAL, "no schedule for these sizes");
    const st::Layout L = st::make_layout(plan1, batch, K, d, n_tasks);  // layout depends on sizes only

    Blob& blob = hs.blob;
    blob.data.clear();
    Groups& ga = groups;
    const size_t at_all_row_off = blob.add(ga.row_off), at_all_rows = blob.add(ga.rows);
    const size_t at_all_q_off = blob.add(ga.q_off), at_all_q = blob.add(ga.q_list);
    const size_t at_q2grp = blob.add(ga.q2grp);
    const SetAt at_m = add_set(blob, set_mfma), at_d = add_set(blob, set_dot);
    const size_t at_blk_off = blob.add(blk_off), at_blk_row = blob.add(blk_row);
    // MFMA scorer: first signature rows of each of its filters (padded with -1), and where the
    // selection kernel stores each query's threshold in the resident-query image
    mp.q_split = std::max(mp.q_split, 1);
    const int32_t rows_local = ((mp.n_blocks + mp.q_split - 1) / mp.q_split) * 16;
    std::vector<int32_t>&prow = hs.prow, &q_taupos = hs.q_taupos;
    prow.assign((size_t)set_mfma.n * st::kPrefetchStride + 1, -1);
    q_taupos.assign((size_t)batch, -1);
    for (int32_t g = 0; g < set_mfma.n; ++g) {
        const int32_t nr = set_mfma.row_off[g + 1] - set_mfma.row_off[g];
        for (int32_t r = 0; r < nr && r < st::kPrefetchStride; ++r)
            prow[(size_t)g * st::kPrefetchStride + r] = set_mfma.rows[set_mfma.row_off[g] + r];
        if (g < st::kMfmaFilterBatch) {
            for (int32_t r = 0; r < nr && r < st::kPrefetchStride; ++r)
                mp.prow_pack[g][r / 4] |= (uint64_t)(uint16_t)set_mfma.rows[set_mfma.row_off[g] + r] << (16 * (r % 4));
            mp.prow_n |= (uint64_t)std::min<int32_t>(nr, st::kPrefetchStride) << (8 * g);
        }
    }
    for (size_t i = 0; i < blk_row.size(); ++i)
        if (blk_row[i] >= 0 && blk_row[i] % n_tasks == 0) {
            const int32_t b = (int32_t)(i / 16), yy = b % mp.q_split, lr = (b / mp.q_split) * 16 + (int32_t)(i % 16);
            q_taupos[blk_row[i] / n_tasks] = yy * (rows_local / n_tasks) + lr / n_tasks;
        }
    if ((size_t)rows_local * mp.q_split > L.img_rows) return fail(ST_EINVAL, "resident-query image too small");
    for (int32_t g = 0; g < set_mfma.n; ++g)
        if ((blk_off[g + 1] - blk_off[g] + mp.q_split - 1) / mp.q_split > 1) mp.multi_block = 1;
    const size_t at_prow = blob.add(prow), at_taupos = blob.add(q_taupos);
    // seed kernel: the first signature rows of every query's filter and their number
    std::vector<int32_t>& q_prow = hs.q_prow;
    q_prow.assign((size_t)batch * (st::kSeedRows + 1), -1);
    for (int32_t b = 0; b < batch; ++b) {
        const int32_t g = groups.q2grp[b], nr = groups.row_off[g + 1] - groups.row_off[g];
        for (int32_t r = 0; r < nr && r < st::kSeedRows; ++r)
            q_prow[(size_t)b * (st::kSeedRows + 1) + r] = groups.rows[groups.row_off[g] + r];
        q_prow[(size_t)b * (st::kSeedRows + 1) + st::kSeedRows] = nr;
    }
    const size_t at_qprow = blob.add(q_prow);
    if (blob.bytes() > L.meta_bytes) return fail(ST_EINVAL, "group tables exceed their workspace slot");
    if (dry_out) {
        dry_out[0] = groups.n_groups;
        dry_out[1] = set_mfma.n;
        dry_out[2] = set_dot.n;
        dry_out[3] = mp.q_split;
        dry_out[4] = set_mfma.n ? mp.waves : 0;
        dry_out[5] = plan.n_levels;
        dry_out[6] = (int32_t)blob.bytes();
        dry_out[7] = plan.n_levels > 0 && plan.level[0].seed ? 1 : 0;
        return ST_OK;
    }

    char* ws = (char*)dev_workspace;
    StageHold stage;
    rc = stage_get(blob.bytes(), stream, &stage);
    if (rc != ST_OK) return rc;
    memcpy(stage.host(), blob.data.data(), blob.bytes());
    // A search that starts with the seed pass lets that kernel bring the tables over (it reads its
    // own from the pinned copy); otherwise they are copied ahead of the first kernel.
    const bool seed_uploads = plan.n_levels > 0 && plan.level[0].seed;
    if (!seed_uploads) {
        stage.enqueued = true;
        ST_HIP(hipMemcpyAsync(ws + L.meta, stage.host(), blob.bytes(), hipMemcpyHostToDevice, stream));
        rc = stage_record(&stage);
        if (rc != ST_OK) return rc;
    }
    auto tab = [&](size_t at) { return (const int32_t*)(ws + L.meta + at); };

    st::ScanParams sp;
    memset(&sp, 0, sizeof(sp));
    sp.bloom = expr_groups ? expr_rows : bloom->dev;
    sp.m_bits = expr_groups ? expr_row_count : bloom->m_bits;
    sp.items = dev_items;
    sp.iscale = dev_item_scale;
    sp.n_items = n_items;
    sp.d = d;
    sp.queries = dev_queries;
    sp.qscale = dev_query_scale;
    sp.batch = batch;
    sp.n_tasks = n_tasks;
    sp.weighted = weighted ? 1 : 0;
    for (int t = 0; t < n_tasks && weighted; ++t) sp.w[t] = host_task_weight[t];
    sp.tau = (const uint64_t*)(ws + L.tau);
    sp.cand = (uint64_t*)(ws + L.cand);
    sp.cnt = (uint32_t*)(ws + L.cnt);
    sp.ovf = (uint32_t*)(ws + L.ovf);
    sp.cap = plan.cap;
    sp.groups = plan.groups;

    st::ScanParams sp_m = sp, sp_d = sp, sp_all = sp;
    sp_m.n_groups = set_mfma.n;
    sp_m.grp_row_off = tab(at_m.row_off);
    sp_m.grp_rows = tab(at_m.rows);
    sp_m.grp_q_off = tab(at_m.q_off);
    sp_m.grp_q = tab(at_m.q_list);
    sp_d.n_groups = set_dot.n;
    sp_d.grp_row_off = tab(at_d.row_off);
    sp_d.grp_rows = tab(at_d.rows);
    sp_d.grp_q_off = tab(at_d.q_off);
    sp_d.grp_q = tab(at_d.q_list);
    sp_all.n_groups = ga.n_groups;
    sp_all.grp_row_off = tab(at_all_row_off);
    sp_all.grp_rows = tab(at_all_rows);
    sp_all.grp_q_off = tab(at_all_q_off);
    sp_all.grp_q = tab(at_all_q);
    mp.grp_blk_off = tab(at_blk_off);
    mp.blk_row = tab(at_blk_row);
    mp.prow = tab(at_prow);
    mp.img_q = (int8_t*)(ws + L.img_q);
    mp.img_sq = (float*)(ws + L.img_sq);
    mp.img_qrow = (int32_t*)(ws + L.img_qrow);
    mp.img_tau = (uint64_t*)(ws + L.img_tau);

    st::SelectParams se;
    memset(&se, 0, sizeof(se));
    se.cand = sp.cand;
    se.cnt = sp.cnt;
    se.cap = plan.cap;
    se.groups = plan.groups;
    se.topk_keys = (uint64_t*)(ws + L.topk_keys);
    se.topk_cnt = (uint32_t*)(ws + L.topk_cnt);
    se.gath = (uint64_t*)(ws + L.gath);
    se.gath_cap = L.gath_cap;
    se.srt = L.k_pad > st::kLdsSortMax ? (uint64_t*)(ws + L.srt) : nullptr;
    se.K = K;
    se.k_pad = L.k_pad;
    // more queries than compute units: a smaller key buffer lets two selection workgroups share one
    se.lds_keys = batch > st::kComputeUnits ? st::kLdsKeysDense : st::kLdsKeys;
    se.tau = (uint64_t*)(ws + L.tau);
    se.ovf = sp.ovf;
    se.out_ids = dev_out_ids;
    se.out_scores = dev_out_scores;
    se.out_count = dev_out_count;

    se.scan = sp_all;
    se.q2grp = tab(at_q2grp);
    se.tau_img = set_mfma.n ? mp.img_tau : nullptr;
    se.q_taupos = tab(at_taupos);
    se.q_prow = tab(at_qprow);
    // Sample mode: the first level of a search that the 8-wavefront MFMA scan serves alone scans
    // its G * cap items as segments spread evenly over the corpus instead of a prefix, and the
    // second level scans the whole corpus without them.  The threshold the first selection
    // publishes rests on the assumption that the order of the corpus says nothing about a query's
    // scores; a strided sample keeps that true for corpora ordered along some trend (by age, by
    // popularity, by category), where a prefix would not.
    int64_t samp_stride = 0;
    if (plan.n_levels >= 2 && !plan.level[0].seed && allow_seed && set_mfma.n && !set_dot.n && mp.waves == 8) {
        const st::Level& L0 = plan.level[0];
        const int64_t segs = (L0.end - L0.begin) / L0.seg_items;
        if (L0.begin == 0 && segs > 0 && (L0.end - L0.begin) % L0.seg_items == 0 && L0.seg_items % 64 == 0) {
            const int64_t stride = n_items / segs / 64 * 64;
            if (stride >= 2 * (int64_t)L0.seg_items) samp_stride = stride;
        }
    }
    bool mfma_started = false;  // the first MFMA launch builds the resident-query image
    bool density_on = false;    // the first level counts the pairs it admits (chooses the later levels' form of the scan)
    int seed_parts = 1;         // slices per query of the seed pass (one threshold each)
    for (int lv = 0; lv < plan.n_levels; ++lv) {
        const st::Level& L_ = plan.level[lv];
        se.first = lv == 0 || (lv == 1 && plan.level[0].seed);  // no candidate list from before
        se.last = lv == plan.n_levels - 1;
        se.may_overflow = lv > 0;
        se.keep = se.last ? K : L_.keep;
        se.keep_prev = lv > 0 ? plan.level[lv - 1].keep : K;
        se.tau_parts = lv == 0 ? 0 : ((lv == 1 && plan.level[0].seed) ? seed_parts : 1);
        if (L_.seed) {  // per-query scan + selection of the prefix in one launch
            TimedLaunch t(1, stream);
            st::SeedUpload up;
            up.src = (const int32_t*)stage.dev_view();
            up.dst = (int32_t*)(ws + L.meta);
            up.words = (int32_t)(blob.bytes() / 4);
            up.img_q = nullptr;
            {  // the words of the pass, spread evenly over the corpus (whole words only)
                const int64_t pass_words = L_.end / 64, all_words = n_items / 64;
                up.word_stride = (L_.end % 64 == 0 && pass_words > 0 && all_words >= 2 * pass_words) ? (int32_t)(all_words / pass_words) : 1;
            }
            if (set_mfma.n) {  // the seed pass stages the scorer's query image as well
                up.img_q = mp.img_q;
                up.img_sq = mp.img_sq;
                up.img_qrow = mp.img_qrow;
                up.blk_row = (const int32_t*)((const char*)stage.dev_view() + at_blk_row);
                up.n_blocks = mp.n_blocks;
                up.q_split = mp.q_split;
                up.rows_local = rows_local;
                mfma_started = true;
            }
            st::SelectParams se_seed = se;  // the seed pass reads its tables from the pinned copy
            auto host_tab = [&](size_t at) { return (const int32_t*)((const char*)stage.dev_view() + at); };
            se_seed.q_prow = host_tab(at_qprow);
            se_seed.q2grp = host_tab(at_q2grp);
            se_seed.q_taupos = host_tab(at_taupos);
            se_seed.scan.grp_row_off = host_tab(at_all_row_off);
            se_seed.scan.grp_rows = host_tab(at_all_rows);
            seed_parts = st::seed_parts(batch, L.k_pad);
            stage.enqueued = true;
            ST_HIP(st::launch_seed(se_seed, L_.end, batch, seed_parts, up, stream));
            rc = stage_record(&stage);
            if (rc != ST_OK) return rc;
            continue;
        }
        for (st::ScanParams* q : {&sp_m, &sp_d}) {
            q->item_begin = (samp_stride && lv == 1) ? 0 : L_.begin;
            q->item_end = L_.end;
            q->samp_role = samp_stride ? (lv == 0 ? 1 : 2) : 0;
            q->samp_stride_items = samp_stride;
            q->samp_segs = samp_stride ? (int32_t)((plan.level[0].end - plan.level[0].begin) / plan.level[0].seg_items) : 0;
            q->samp_seg_items = samp_stride ? plan.level[0].seg_items : 0;
            q->seg_items = L_.seg_items;
            q->seg_per_visit = L_.seg_per_visit;
            q->use_tau = lv > 0;
            q->tau_parts = (lv == 1 && plan.level[0].seed) ? seed_parts : 1;
        }
        const int64_t n_seg = (L_.end - sp_m.item_begin + L_.seg_items - 1) / L_.seg_items;
        // workgroups of the MFMA scan that are resident at once, per row of the grid
        const int32_t resident = std::max(1, st::pow2_ceil(st::kComputeUnits * mfma_wgs / mp.q_split + 1) / 2);
        // Past the first level a visit is one segment per wavefront of the workgroup; a level with
        // fewer segments than that gives every resident workgroup takes shorter visits instead, so
        // that all of them (and with them all of their candidate regions) take part.
        if (lv > 0 && mp.waves > L_.seg_per_visit) {
            sp_m.seg_per_visit = mp.waves;
            // (with the second scorer in the same search every region has its own workgroup)
            const int64_t wgs = set_dot.n ? plan.groups / mp.q_split : resident;
            if (set_mfma.n && n_seg < wgs * mp.waves)
                sp_m.seg_per_visit = (int32_t)std::max<int64_t>(1, (n_seg + wgs - 1) / wgs);
        }
        // the same for the wavefront-dot scorer, whose workgroups take a visit's segments in turn
        if (lv > 0 && n_seg < (int64_t)plan.groups * L_.seg_per_visit)
            sp_d.seg_per_visit = (int32_t)std::max<int64_t>(1, (n_seg + plan.groups - 1) / plan.groups);
        // workgroups with work: one visit (seg_per_visit segments) per step; launching no more
        // keeps idle workgroups from staging queries, and the selection reads only their regions
        const int64_t n_visit = (n_seg + sp_m.seg_per_visit - 1) / sp_m.seg_per_visit;
        int32_t regions = plan.groups;
        if (set_mfma.n) {
            const int32_t per_row = plan.groups / mp.q_split;  // regions of one row of the grid
            int32_t gx = per_row;
            mp.region_slots = 1;
            if (!set_dot.n) {
                // only as many workgroups as are resident at once; each takes several regions
                if (resident < gx) gx = resident;
                if (n_visit < gx) gx = (int32_t)std::max<int64_t>(n_visit, 1);
                // the first level needs exactly one visit per region; later levels spread each
                // workgroup's candidates, segment by segment, over the regions the layout leaves it
                // (as many as the LDS budget of the chosen configuration was sized for)
                const int64_t want = lv == 0 ? std::min<int64_t>(per_row / gx, (n_visit + gx - 1) / gx)
                                             : std::min<int64_t>(per_row / gx, st::mfma_region_slots(mfma_wgs));
                mp.region_slots = (int32_t)std::max<int64_t>(1, std::min<int64_t>(want, st::kMaxRegionSlots));
                // the first level needs a region per visit (no region can then overflow)
                if (lv == 0 && (int64_t)gx * mp.region_slots < n_visit) {
                    gx = (int32_t)std::min<int64_t>(per_row, std::max<int64_t>(n_visit, 1));
                    mp.region_slots = 1;
                }
            }
            regions = set_dot.n ? plan.groups : gx * mp.region_slots * mp.q_split;
            st::mfma_lds_layout(&mp, d, n_tasks, set_mfma.n, mp.waves);
            mp.first_level = mfma_started ? 0 : 1;
            // A first level that admits every pair also counts them: the later levels choose the
            // form of the scan by how many items a filter passes per segment.
            {
                st::ScanParams probe = sp_m;
                probe.use_tau = lv > 0;
                const bool admit_all = lv == 0 && mp.waves == 8 && !set_dot.n && probe.seg_per_visit == 1 && probe.seg_items <= probe.cap;
                if (lv == 0) {
                    density_on = admit_all;
                    mp.density_acc = admit_all ? (unsigned long long*)(ws + L.density) : nullptr;
                    // pairs of the level if every filter passed kDenseItems items per 512-item segment
                    mp.density_limit = (unsigned long long)((L_.end - L_.begin) * (int64_t)batch / 512 * st::kDenseItems);
                } else if (!density_on) {
                    mp.density_acc = nullptr;
                }
            }
            mfma_started = true;
            TimedLaunch t(0, stream);
            ST_HIP(st::launch_scan_mfma(sp_m, mp, gx, stream));
        }
        if (set_dot.n) {
            TimedLaunch t(0, stream);
            hipLaunchKernelGGL(st::scan_wavedot_kernel, dim3(plan.groups), dim3(st::kScanThreads),
                               (size_t)((batch + 1) & ~1) * 4 + (size_t)batch * 8, stream, sp_d);
            ST_HIP(hipGetLastError());
        }
        se.regions = regions;
        se.density_acc = (lv == 0 && density_on) ? (unsigned long long*)(ws + L.density) : nullptr;
        {
            TimedLaunch t(1, stream);
            // K above the LDS sort size: the final ordering of k_pad keys runs in LDS where they fit
            const size_t big_bytes = (size_t)L.k_pad * 8;
            constexpr size_t kBigSortMax = 128 * 1024;
            se.big_sort = se.srt ? (big_bytes <= kBigSortMax ? 1 : 2) : 0;
            static std::atomic<bool> lds_set{false};  // (setting the attribute twice is harmless)
            if (!lds_set.load(std::memory_order_acquire)) {
                ST_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&st::select_kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize,
                                           (int)std::max<size_t>(st::kSelectLdsBytes, kBigSortMax)));
                lds_set.store(true, std::memory_order_release);
            }
            const size_t lds = std::max<size_t>((size_t)st::select_lds_bytes(se.lds_keys), se.big_sort == 1 ? big_bytes : (se.big_sort == 2 ? kBigSortMax : 0));
            hipLaunchKernelGGL(st::select_kernel, dim3(batch), dim3(st::kSelectThreads), lds, stream, se);
        }
        ST_HIP(hipGetLastError());
    }
    return ST_OK;
}

int st_search(const st_bloom* bloom, const int8_t* dev_items, const float* dev_item_scale, int64_t n_items,
              int32_t d, const int8_t* dev_queries, const float* dev_query_scale, int32_t batch,
              const uint64_t* host_filt_ids, const int64_t* host_filt_offsets, int32_t K,
              int64_t* dev_out_ids, float* dev_out_scores, int32_t* dev_out_count, void* dev_workspace,
              int64_t workspace_bytes, void* hip_stream)
{
    return guarded([&]() -> int {
    return search_impl(bloom, dev_items, dev_item_scale, n_items, d, dev_queries, dev_query_scale, batch, 1,
                       nullptr, host_filt_ids, host_filt_offsets, K, dev_out_ids, dev_out_scores,
                       dev_out_count, dev_workspace, workspace_bytes, hip_stream);
    });
}

int st_search_static(const st_bloom* bloom, const int8_t* dev_items, const float* dev_item_scale, int64_t n_items,
                     int32_t d, const int8_t* dev_queries, const float* dev_query_scale, int32_t batch,
                     const uint64_t* host_filt_ids, const int64_t* host_filt_offsets, int32_t K,
                     int64_t* dev_out_ids, float* dev_out_scores, int32_t* dev_out_count, void* hip_stream)
{
    return guarded([&]() -> int {
        if (!bloom) return fail(ST_EINVAL, "bloom is null");
        const int64_t need = st_search_workspace_bytes(n_items, d, batch, 1, K);
        if (need < 0) return (int)need;
        if (need > (int64_t)ST_STATIC_SCRATCH_BYTES)
            return fail(ST_EWORKSPACE, "these sizes need %lld bytes of workspace, the static one holds %lld: use st_search",
                        (long long)need, (long long)ST_STATIC_SCRATCH_BYTES);
        int device = -1;
        ST_HIP(hipGetDevice(&device));
        if (device != bloom->device) return fail(ST_EINVAL, "the index lives on device %d, the current device is %d", bloom->device, device);
        void* ws = device >= 0 && device < kMaxDevices ? g_scratch_ptr[device] : nullptr;
        if (!ws) return fail(ST_EINVAL, "no static workspace on device %d (st_bloom_build sets it up)", device);
        struct NoAlloc {
            NoAlloc() { t_no_alloc = true; }
            ~NoAlloc() { t_no_alloc = false; }
        } guard;
        return search_impl(bloom, dev_items, dev_item_scale, n_items, d, dev_queries, dev_query_scale, batch, 1,
                           nullptr, host_filt_ids, host_filt_offsets, K, dev_out_ids, dev_out_scores, dev_out_count,
                           ws, (int64_t)ST_STATIC_SCRATCH_BYTES, hip_stream);
    });
}

int st_search_multitask(const st_bloom* bloom, const int8_t* dev_items, const float* dev_item_scale,
                        int64_t n_items, int32_t d, const int8_t* dev_queries, const float* dev_query_scale,
                        int32_t batch, int32_t n_tasks, const float* host_task_weight,
                        const uint64_t* host_filt_ids, const int64_t* host_filt_offsets, int32_t K,
                        int64_t* dev_out_ids, float* dev_out_scores, int32_t* dev_out_count,
                        void* dev_workspace, int64_t workspace_bytes, void* hip_stream)
{
    return guarded([&]() -> int {
    if (!host_task_weight) return fail(ST_EINVAL, "host_task_weight is null");
    return search_impl(bloom, dev_items, dev_item_scale, n_items, d, dev_queries, dev_query_scale, batch,
                       n_tasks, host_task_weight, host_filt_ids, host_filt_offsets, K, dev_out_ids,
                       dev_out_scores, dev_out_count, dev_workspace, workspace_bytes, hip_stream);
    });
}

int st_search_host_plan(int64_t n_items, int32_t d, int32_t batch, int32_t n_tasks, int32_t K, int32_t m_bits,
                        int32_t k_hashes, const uint64_t* host_filt_ids, const int64_t* host_filt_offsets,
                        int32_t* host_out_summary)
{
    return guarded([&]() -> int {
        if (!host_out_summary) return fail(ST_EINVAL, "host_out_summary is null");
        if (m_bits < 1 || m_bits > ST_MAX_M_BITS) return fail(ST_EINVAL, "m_bits=%d out of range", m_bits);
        if (k_hashes < 1 || k_hashes > ST_MAX_K_HASHES) return fail(ST_EINVAL, "k_hashes=%d out of range", k_hashes);
        st_bloom desc;  // sizes only: the dry run reads no device memory
        desc.n_items = n_items;
        desc.m_bits = m_bits;
        desc.k_hashes = k_hashes;
        const float unit_weights[ST_MAX_TASKS] = {1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f, 1.f};
        return search_impl(&desc, nullptr, nullptr, n_items, d, nullptr, nullptr, batch, n_tasks,
                           n_tasks > 1 ? unit_weights : nullptr, host_filt_ids, host_filt_offsets, K, nullptr, nullptr,
                           nullptr, nullptr, 0, nullptr, nullptr, nullptr, 0, true, 64, host_out_summary);
    });
}

int st_bloom_mask_expr(const st_bloom* bloom, const int32_t* host_expr_ops, const uint64_t* host_expr_ids,
                       const int64_t* host_expr_offsets, int32_t n_exprs, uint64_t* dev_mask, void* hip_stream)
{
    return guarded([&]() -> int {
    if (!bloom || !host_expr_offsets || !dev_mask) return fail(ST_EINVAL, "null argument");
    if (n_exprs < 0 || n_exprs > 65535) return fail(ST_EINVAL, "n_exprs=%d out of range", n_exprs);
    ExprTables tab;
    int rc = build_programs(host_expr_ops, host_expr_ids, host_expr_offsets, n_exprs, bloom->m_bits, bloom->k_hashes,
                            &tab, nullptr);
    if (rc != ST_OK) return rc;
    if (n_exprs == 0 || bloom->n_items == 0) return ST_OK;
    hipStream_t stream = (hipStream_t)hip_stream;
    tab.code.push_back(0);       // (never empty, so that data() is a real address)
    tab.leaf_rows.push_back(0);
    int32_t* d_tab = nullptr;
    const size_t n_off = tab.prog_off.size(), n_code = tab.code.size(), n_rows = tab.leaf_rows.size();
    ST_HIP(hipMalloc((void**)&d_tab, (n_off + n_code + n_rows) * 4));
    auto body = [&]() -> int {
        ST_HIP(hipMemcpyAsync(d_tab, tab.prog_off.data(), n_off * 4, hipMemcpyHostToDevice, stream));
        ST_HIP(hipMemcpyAsync(d_tab + n_off, tab.code.data(), n_code * 4, hipMemcpyHostToDevice, stream));
        ST_HIP(hipMemcpyAsync(d_tab + n_off + n_code, tab.leaf_rows.data(), n_rows * 4, hipMemcpyHostToDevice, stream));
        const int64_t n_words = (bloom->n_items + 63) / 64;
        dim3 grid((unsigned)((n_words + 255) / 256), (unsigned)n_exprs);
        hipLaunchKernelGGL(st::bloom_expr_kernel, grid, dim3(256), 0, stream, bloom->dev, bloom->m_bits,
                           bloom->k_hashes, bloom->n_items, n_words, d_tab, d_tab + n_off, d_tab + n_off + n_code, 0,
                           dev_mask);
        ST_HIP(hipGetLastError());
        ST_HIP(hipStreamSynchronize(stream));
        return ST_OK;
    };
    rc = body();
    (void)hipFree(d_tab);
    return rc;
    });
}

static int64_t expr_ws_bytes(int64_t n_items, int32_t d, int32_t batch, int32_t n_tasks, int32_t K,
                             int64_t n_expr_entries, int32_t min_cap)
{
    const int64_t base = search_ws_bytes(n_items, d, batch, n_tasks, K, min_cap);
    if (base < 0) return base;
    if (n_expr_entries < 0 || n_expr_entries > (int64_t)batch * ST_MAX_EXPR_OPS)
        return fail(ST_EINVAL, "n_expr_entries=%lld out of range", (long long)n_expr_entries);
    const int64_t n_tiles = (n_items + st::kTileItems - 1) / st::kTileItems;
    // the search's own workspace, one mask row per query (every program distinct), the tables
    return st::round_up(base, 256) + n_tiles * batch * st::kTileWords * 8 +
           (int64_t)expr_table_bytes(batch, n_expr_entries, ST_MAX_K_HASHES);
}

int64_t st_search_expr_workspace_bytes(int64_t n_items, int32_t d, int32_t batch, int32_t n_tasks, int32_t K,
                                       int64_t n_expr_entries)
{
    return expr_ws_bytes(n_items, d, batch, n_tasks, K, n_expr_entries, 64);
}

int st_search_expr(const st_bloom* bloom, const int8_t* dev_items, const float* dev_item_scale, int64_t n_items,
                   int32_t d, const int8_t* dev_queries, const float* dev_query_scale, int32_t batch,
                   int32_t n_tasks, const float* host_task_weight, const int32_t* host_expr_ops,
                   const uint64_t* host_expr_ids, const int64_t* host_expr_offsets, int32_t K,
                   int64_t* dev_out_ids, float* dev_out_scores, int32_t* dev_out_count, void* dev_workspace,
                   int64_t workspace_bytes, void* hip_stream)
{
    return guarded([&]() -> int {
    if (!bloom || !host_expr_offsets || !dev_workspace) return fail(ST_EINVAL, "null argument");
    if (!host_task_weight && n_tasks != 1) return fail(ST_EINVAL, "n_tasks=%d needs host_task_weight", n_tasks);
    const int64_t base = st_search_workspace_bytes(n_items, d, batch, n_tasks, K);
    if (base < 0) return (int)base;
    if (n_items != bloom->n_items)
        return fail(ST_EINVAL, "n_items=%lld but the index holds %lld", (long long)n_items, (long long)bloom->n_items);
    if ((uintptr_t)dev_workspace & 255) return fail(ST_EINVAL, "misaligned workspace (256 B)");
    ExprTables tab;
    Groups groups;
    int rc = build_programs(host_expr_ops, host_expr_ids, host_expr_offsets, batch, bloom->m_bits, bloom->k_hashes,
                            &tab, &groups);
    if (rc != ST_OK) return rc;
    const int64_t need = st_search_expr_workspace_bytes(n_items, d, batch, n_tasks, K, host_expr_offsets[batch]);
    if (need < 0) return (int)need;
    if (workspace_bytes < need)
        return fail(ST_EWORKSPACE, "workspace has %lld bytes, %lld needed", (long long)workspace_bytes, (long long)need);
    hipStream_t stream = (hipStream_t)hip_stream;
    const int64_t n_tiles = (n_items + st::kTileItems - 1) / st::kTileItems;
    char* ws = (char*)dev_workspace;
    uint64_t* mask_rows = (uint64_t*)(ws + st::round_up(base, 256));
    int32_t* d_tab = (int32_t*)((char*)mask_rows + n_tiles * batch * st::kTileWords * 8);

    if (n_tiles > 0) {
        // tables through a pinned slot (asynchronous copy), then one launch evaluates every
        // distinct program into its row of the mask index
        const size_t n_off = tab.prog_off.size(), n_code = tab.code.size(), n_rows = tab.leaf_rows.size();
        const size_t bytes = (n_off + n_code + n_rows) * 4;
        if (bytes > expr_table_bytes(batch, host_expr_offsets[batch], ST_MAX_K_HASHES))
            return fail(ST_EINVAL, "program tables exceed their workspace slot");
        StageHold stage;
        rc = stage_get(bytes, stream, &stage);
        if (rc != ST_OK) return rc;
        int32_t* h = (int32_t*)stage.host();
        memcpy(h, tab.prog_off.data(), n_off * 4);
        if (n_code) memcpy(h + n_off, tab.code.data(), n_code * 4);
        if (n_rows) memcpy(h + n_off + n_code, tab.leaf_rows.data(), n_rows * 4);
        // small tables are read by the kernel straight from the pinned slot (each workgroup fetches
        // its program once); larger ones are copied to the workspace first
        const int32_t* t_dev = (const int32_t*)stage.dev_view();
        stage.enqueued = true;
        if (bytes > 64 * 1024) {
            ST_HIP(hipMemcpyAsync(d_tab, stage.host(), bytes, hipMemcpyHostToDevice, stream));
            t_dev = d_tab;
        }
        const int64_t n_words = n_tiles * st::kTileWords;  // whole tiles: the pad words become 0
        dim3 grid((unsigned)((n_words + 255) / 256), (unsigned)tab.n_exprs);
        {
            TimedLaunch t(3, stream);
            hipLaunchKernelGGL(st::bloom_expr_kernel, grid, dim3(256), 0, stream, bloom->dev, bloom->m_bits,
                               bloom->k_hashes, n_items, n_words, t_dev, t_dev + n_off, t_dev + n_off + n_code,
                               tab.n_exprs, mask_rows);
        }
        ST_HIP(hipGetLastError());
        rc = stage_record(&stage);
        if (rc != ST_OK) return rc;
    }
    return search_impl(bloom, dev_items, dev_item_scale, n_items, d, dev_queries, dev_query_scale, batch, n_tasks,
                       host_task_weight, nullptr, nullptr, K, dev_out_ids, dev_out_scores, dev_out_count,
                       dev_workspace, base, hip_stream, &groups, mask_rows, tab.n_exprs);
    });
}

// Region capacity of the probing search: the largest, so that the first level (every pair
// admitted) is long enough to give every query a threshold although its passing items sit in a few
// item ranges, and a dense range cannot overflow a region.
static constexpr int32_t kIvfCap = 512;

int64_t st_search_ivf_workspace_bytes(int64_t n_items, int32_t d, int32_t batch, int32_t K, int32_t n_clusters,
                                      int32_t n_probe, int64_t n_expr_entries)
{
    const int64_t base = expr_ws_bytes(n_items, d, batch, 1, K, n_expr_entries, kIvfCap);
    if (base < 0) return base;
    if (n_clusters < 1 || n_clusters > ST_MAX_CLUSTERS) return fail(ST_EINVAL, "n_clusters=%d out of range", n_clusters);
    if (n_probe < 1 || n_probe > ST_MAX_PROBES) return fail(ST_EINVAL, "n_probe=%d out of range", n_probe);
    // centroid keys and probed cluster ids behind the expression search's workspace
    return st::round_up(base, 256) + st::round_up((int64_t)batch * n_clusters * 8, 256) +
           st::round_up((int64_t)batch * n_probe * 4, 256) +
           st::round_up((int64_t)batch * (st::kQueryParts + st::kProbeParts) * 4, 256);
}

int st_search_ivf(const st_bloom* bloom, const int8_t* dev_items, const float* dev_item_scale, int64_t n_items,
                  int32_t d, const int8_t* dev_centroids, const float* dev_centroid_scale,
                  const int64_t* dev_cluster_offsets, int32_t n_clusters, int32_t n_probe,
                  const int8_t* dev_queries, const float* dev_query_scale, int32_t batch,
                  const int32_t* host_expr_ops, const uint64_t* host_expr_ids, const int64_t* host_expr_offsets,
                  int32_t K, int64_t* dev_out_ids, float* dev_out_scores, int32_t* dev_out_count,
                  int32_t* dev_out_probes, void* dev_workspace, int64_t workspace_bytes, void* hip_stream)
{
    return guarded([&]() -> int {
    if (!bloom || !host_expr_offsets || !dev_workspace || !dev_centroids || !dev_centroid_scale ||
        !dev_cluster_offsets || !dev_queries || !dev_query_scale)
        return fail(ST_EINVAL, "null argument");
    const int64_t base = search_ws_bytes(n_items, d, batch, 1, K, kIvfCap);
    if (base < 0) return (int)base;
    if (n_items != bloom->n_items)
        return fail(ST_EINVAL, "n_items=%lld but the index holds %lld", (long long)n_items, (long long)bloom->n_items);
    if (((uintptr_t)dev_workspace & 255) || ((uintptr_t)dev_centroids & 15) || ((uintptr_t)dev_queries & 15))
        return fail(ST_EINVAL, "misaligned buffer (workspace 256 B; centroids and queries 16 B)");
    ExprTables tab;
    int rc = build_programs(host_expr_ops, host_expr_ids, host_expr_offsets, batch, bloom->m_bits, bloom->k_hashes,
                            &tab, nullptr);  // one program per query, in order
    if (rc != ST_OK) return rc;
    const int64_t expr_ws = expr_ws_bytes(n_items, d, batch, 1, K, host_expr_offsets[batch], kIvfCap);
    const int64_t need = st_search_ivf_workspace_bytes(n_items, d, batch, K, n_clusters, n_probe, host_expr_offsets[batch]);
    if (need < 0) return (int)need;
    if (workspace_bytes < need)
        return fail(ST_EWORKSPACE, "workspace has %lld bytes, %lld needed", (long long)workspace_bytes, (long long)need);
    hipStream_t stream = (hipStream_t)hip_stream;
    const int64_t n_tiles = (n_items + st::kTileItems - 1) / st::kTileItems;
    char* ws = (char*)dev_workspace;
    uint64_t* mask_rows = (uint64_t*)(ws + st::round_up(base, 256));
    int32_t* d_tab = (int32_t*)((char*)mask_rows + n_tiles * batch * st::kTileWords * 8);
    char* tail = ws + st::round_up(expr_ws, 256);

    st::IvfParams ip;
    memset(&ip, 0, sizeof(ip));
    ip.queries = dev_queries;
    ip.qscale = dev_query_scale;
    ip.centroids = dev_centroids;
    ip.cscale = dev_centroid_scale;
    ip.cluster_off = dev_cluster_offsets;
    ip.d = d;
    ip.n_clusters = n_clusters;
    ip.n_probe = n_probe;
    ip.k_pad = st::pow2_ceil(std::min(n_probe, n_clusters));
    ip.batch = batch;
    ip.n_items = n_items;
    ip.keys = (uint64_t*)tail;
    ip.probes = (int32_t*)(tail + st::round_up((int64_t)batch * n_clusters * 8, 256));
    ip.user_probes = dev_out_probes;
    uint32_t* q_parts = (uint32_t*)((char*)ip.probes + st::round_up((int64_t)batch * n_probe * 4, 256));  // [batch][kQueryParts]

    // Few enough probes for one workgroup to lay out: phases 2-4 run per query over the probed
    // ranges alone.  (A forced scoring path selects the scan-based route below instead, which also
    // serves larger probe counts.)
    const bool per_query = g_scoring_path == 0 && n_probe <= st::kQueryProbes;
    if (per_query) {
        if (!dev_out_ids || !dev_out_scores || !dev_out_count || (n_items > 0 && (!dev_items || !dev_item_scale)))
            return fail(ST_EINVAL, "null argument");
        if (((uintptr_t)dev_items & 15) || ((uintptr_t)dev_item_scale & 3))
            return fail(ST_EINVAL, "misaligned buffer (items 16 B)");
    }

    // every query is its own filter group: its probed clusters are its own
    Groups groups;
    groups.n_groups = batch;
    groups.row_off.assign(1, 0);
    groups.q_off.assign(1, 0);
    for (int32_t b = 0; b < batch; ++b) {
        groups.rows.push_back(b);
        groups.row_off.push_back(b + 1);
        groups.q_list.push_back(b);
        groups.q_off.push_back(b + 1);
        groups.q2grp.push_back(b);
    }

    {   // phase 1: centroid scores and the n_probe best clusters of every query
        // Many centroids: several workgroups per query, each on a slice, then a merge.  The number of
        // parts is the largest that keeps a slice within the register-resident select and all parts'
        // survivors within the merge's.
        int parts = 1, chunk = n_clusters;
        if (n_clusters >= 4096)
            for (int pp = st::kProbeParts; pp >= 2; pp >>= 1) {
                const int ch = (n_clusters + pp - 1) / pp;
                if (ch <= st::kTopkRegs * st::kProbeThreads &&
                    (int64_t)pp * std::min(n_probe, ch) <= (int64_t)st::kTopkRegs * st::kProbeMergeThreads) {
                    parts = pp;
                    chunk = ch;
                    break;
                }
            }
        TimedLaunch t(3, stream);
        if (parts > 1) {
            uint32_t* probe_cnt = q_parts + (size_t)batch * st::kQueryParts;  // [batch][kProbeParts]
            hipLaunchKernelGGL(st::ivf_probe_part_kernel, dim3(batch, parts), dim3(st::kProbeThreads), 0, stream, ip, chunk,
                               probe_cnt);
            hipLaunchKernelGGL(st::ivf_probe_merge_kernel, dim3(batch), dim3(st::kProbeMergeThreads), 0, stream, ip, chunk,
                               parts, probe_cnt);
        } else {
            hipLaunchKernelGGL(st::ivf_probe_kernel, dim3(batch), dim3(st::kProbeThreads), st::probe_lds_bytes(ip.k_pad),
                               stream, ip);
        }
    }
    ST_HIP(hipGetLastError());
    if (n_tiles > 0) {
        const size_t n_off = tab.prog_off.size(), n_code = tab.code.size(), n_rows = tab.leaf_rows.size();
        const size_t bytes = (n_off + n_code + n_rows) * 4;
        if (bytes > expr_table_bytes(batch, host_expr_offsets[batch], ST_MAX_K_HASHES))
            return fail(ST_EINVAL, "program tables exceed their workspace slot");
        StageHold stage;
        rc = stage_get(bytes, stream, &stage);
        if (rc != ST_OK) return rc;
        int32_t* h = (int32_t*)stage.host();
        memcpy(h, tab.prog_off.data(), n_off * 4);
        if (n_code) memcpy(h + n_off, tab.code.data(), n_code * 4);
        if (n_rows) memcpy(h + n_off + n_code, tab.leaf_rows.data(), n_rows * 4);
        const int32_t* t_dev = (const int32_t*)stage.dev_view();
        stage.enqueued = true;
        if (bytes > 64 * 1024) {
            ST_HIP(hipMemcpyAsync(d_tab, stage.host(), bytes, hipMemcpyHostToDevice, stream));
            t_dev = d_tab;
        }
        if (per_query) {
            st::Plan plan1;
            if (cached_plan(n_items, K, 1, st::kMaxSegItems, batch, &plan1, 2048, kIvfCap) != 0)
                return fail(ST_EINVAL, "no schedule for these sizes");
            const st::Layout L = st::make_layout(plan1, batch, K, d, 1);
            st::IvfQueryParams qp;
            memset(&qp, 0, sizeof(qp));
            qp.ivf = ip;
            qp.bloom = bloom->dev;
            qp.m_bits = bloom->m_bits;
            qp.k_hashes = bloom->k_hashes;
            qp.items = dev_items;
            qp.iscale = dev_item_scale;
            qp.prog_off = t_dev;
            qp.code = t_dev + n_off;
            qp.leaf_rows = t_dev + n_off + n_code;
            qp.gath = (uint64_t*)(ws + L.gath);
            qp.gath_cap = L.gath_cap;
            qp.srt = L.k_pad > st::kLdsSortMax ? (uint64_t*)(ws + L.srt) : nullptr;
            qp.K = K;
            qp.k_pad = L.k_pad;
            qp.out_ids = dev_out_ids;
            qp.out_scores = dev_out_scores;
            qp.out_count = dev_out_count;
            qp.ovf = (uint32_t*)(ws + L.ovf);
            qp.part_cnt = q_parts;
            // Workgroups per query: enough to occupy the chip, as long as every part's share of the
            // key buffer holds a round beside the K keys it keeps, the parts' survivors fit the final
            // selection in LDS together, and the result is sorted in LDS.
            int parts = 1;
            if (!qp.srt) {
                auto fits = [&](int pp) {
                    return pp <= st::kQueryParts && (int64_t)pp * K <= (int64_t)st::kTopkRegs * st::kQueryThreads &&
                           L.gath_cap / pp >= 2 * (int64_t)K + 64 * st::kQueryThreads;
                };
                while (fits(parts * 2) && batch * parts * 2 <= st::kComputeUnits) parts *= 2;
                // a large batch fills the chip by itself, but queries with many probed words still gain
                // from parts (the longest query sets the kernel's duration): two rounds per part at least
                const int64_t words = (int64_t)n_probe * (n_items / std::max(n_clusters, 1) / 64 + 1);
                while (fits(parts * 2) && words / parts > 2 * st::kQueryThreads) parts *= 2;
            }
            {
                TimedLaunch t(0, stream);
                hipLaunchKernelGGL(st::ivf_query_kernel, dim3(batch, parts), dim3(st::kQueryThreads), 0, stream, qp);
                if (parts > 1)
                    hipLaunchKernelGGL(st::ivf_merge_kernel, dim3(batch), dim3(st::kQueryThreads), 0, stream, qp, parts);
            }
            ST_HIP(hipGetLastError());
            return stage_record(&stage);
        }
        {   // phase 2: the filter over the probed ranges only, into zeroed mask rows
            TimedLaunch t(3, stream);
            const int64_t n_mask_words = n_tiles * batch * st::kTileWords;
            hipLaunchKernelGGL(st::fill_zero_kernel, dim3((unsigned)std::min<int64_t>((n_mask_words + 255) / 256, 4096)),
                               dim3(256), 0, stream, mask_rows, n_mask_words);
            hipLaunchKernelGGL(st::ivf_mask_kernel, dim3((unsigned)((n_probe + st::kMaskProbes - 1) / st::kMaskProbes), (unsigned)batch), dim3(256), 0, stream,
                               bloom->dev, bloom->m_bits, bloom->k_hashes, ip, t_dev, t_dev + n_off,
                               t_dev + n_off + n_code, mask_rows);
        }
        ST_HIP(hipGetLastError());
        rc = stage_record(&stage);
        if (rc != ST_OK) return rc;
    }
    // phases 3 and 4
    return search_impl(bloom, dev_items, dev_item_scale, n_items, d, dev_queries, dev_query_scale, batch, 1, nullptr,
                       nullptr, nullptr, K, dev_out_ids, dev_out_scores, dev_out_count, dev_workspace, base,
                       hip_stream, &groups, mask_rows, batch, false, kIvfCap);
    });
}

int st_quantize_global(const float* dev_x, int64_t n_rows, int32_t d, int8_t* dev_q, float* dev_row_scale,
                       float* dev_minmax, void* dev_scratch8, void* hip_stream)
{
    if (n_rows < 0 || d < 1 || d > ST_MAX_DIM || n_rows > (1LL << 40) / d)
        return fail(ST_EINVAL, "bad table size %lld x %d", (long long)n_rows, d);
    if (!dev_minmax || !dev_scratch8 || (n_rows > 0 && (!dev_x || !dev_q || !dev_row_scale)))
        return fail(ST_EINVAL, "null argument");
    if (((uintptr_t)dev_x & 15) || ((uintptr_t)dev_q & 15) || ((uintptr_t)dev_scratch8 & 7))
        return fail(ST_EINVAL, "misaligned buffer (table and output 16 B, scratch 8 B)");
    hipStream_t stream = (hipStream_t)hip_stream;
    const int64_t n = n_rows * d;
    uint32_t* mm = (uint32_t*)dev_scratch8;
    // enough workgroups to fill the chip, each streaming many values
    const unsigned grid = (unsigned)std::max<int64_t>(1, std::min<int64_t>((n / 16 + st::kQuantThreads - 1) / st::kQuantThreads,
                                                                         st::kComputeUnits * 16));
    hipLaunchKernelGGL(st::quant_init_kernel, dim3(1), dim3(64), 0, stream, mm);
    if (n > 0) {
        TimedLaunch t(0, stream);
        hipLaunchKernelGGL(st::quant_minmax_kernel, dim3(grid), dim3(st::kQuantThreads), 0, stream, dev_x, n, mm);
    }
    {
        TimedLaunch t(0, stream);
        hipLaunchKernelGGL(st::quant_apply_kernel, dim3(grid), dim3(st::kQuantThreads), 0, stream, dev_x, n, n_rows, mm,
                           dev_q, dev_row_scale, dev_minmax);
    }
    ST_HIP(hipGetLastError());
    return ST_OK;
}

int st_stream_read(const void* dev_src, int64_t bytes, void* dev_sink, int32_t workgroups, void* hip_stream)
{
    if (!dev_src || !dev_sink || bytes < 0) return fail(ST_EINVAL, "null argument or negative size");
    if (((uintptr_t)dev_src & 15) || ((uintptr_t)dev_sink & 3)) return fail(ST_EINVAL, "misaligned buffer (source 16 B, sink 4 B)");
    if (workgroups < 1 || workgroups > 65536) return fail(ST_EINVAL, "workgroups=%d out of range", workgroups);
    {
        TimedLaunch t(0, (hipStream_t)hip_stream);
        hipLaunchKernelGGL(st::stream_read_kernel, dim3((unsigned)workgroups), dim3(st::kStreamThreads), 0,
                           (hipStream_t)hip_stream, (const int4*)dev_src, bytes / 16, (uint32_t*)dev_sink);
    }
    ST_HIP(hipGetLastError());
    return ST_OK;
}

int st_value_model(const float* dev_task_scores, int64_t n, int32_t n_tasks, const int32_t* host_ops,
                   const float* host_consts, int32_t n_ops, float* dev_out, void* hip_stream)
{
    static_assert(ST_MAX_VM_OPS == st::kVmOps && ST_MAX_VM_DEPTH == st::kVmDepth, "formula limits follow the kernel");
    if (n < 0 || n_tasks < 1 || n_tasks > 64) return fail(ST_EINVAL, "bad sizes");
    if (!host_ops || !host_consts || (n > 0 && (!dev_task_scores || !dev_out))) return fail(ST_EINVAL, "null argument");
    if (n_ops < 1 || n_ops > ST_MAX_VM_OPS) return fail(ST_EINVAL, "formula has %d entries (1 to %d)", n_ops, ST_MAX_VM_OPS);
    st::VmProgram prog;
    memset(&prog, 0, sizeof(prog));
    prog.n_ops = n_ops;
    int depth = 0, deepest = 0;
    for (int32_t i = 0; i < n_ops; ++i) {
        const int32_t code = host_ops[i] & 255;
        switch (code) {
        case ST_VM_TASK:
            if ((host_ops[i] >> 8) < 0 || (host_ops[i] >> 8) >= n_tasks)
                return fail(ST_EINVAL, "formula entry %d names task %d of %d", i, host_ops[i] >> 8, n_tasks);
            ++depth;
            break;
        case ST_VM_CONST:
            if (!std::isfinite(host_consts[i])) return fail(ST_EINVAL, "formula constant %d is not finite", i);
            ++depth;
            break;
        case ST_VM_ADD: case ST_VM_SUB: case ST_VM_MUL: case ST_VM_MIN: case ST_VM_MAX: case ST_VM_GT:
            if (depth < 2) return fail(ST_EINVAL, "formula entry %d lacks operands", i);
            --depth;
            break;
        case ST_VM_SELECT:
            if (depth < 3) return fail(ST_EINVAL, "formula entry %d lacks operands", i);
            depth -= 2;
            break;
        default:
            return fail(ST_EINVAL, "formula entry %d: unknown operation %d", i, code);
        }
        if (depth > ST_MAX_VM_DEPTH) return fail(ST_EINVAL, "formula needs a stack deeper than %d", ST_MAX_VM_DEPTH);
        deepest = std::max(deepest, depth);
        prog.ops[i] = host_ops[i];
        prog.consts[i] = host_consts[i];
    }
    if (depth != 1) return fail(ST_EINVAL, "formula leaves %d results", depth);
    if (n == 0) return ST_OK;
    const int64_t sets = (n + st::kVmItems - 1) / st::kVmItems;  // items of one thread
    const unsigned grid = (unsigned)std::min<int64_t>((sets + st::kVmThreads - 1) / st::kVmThreads, st::kComputeUnits * 16);
    {
        static std::atomic<bool> lds_set{false};  // (setting the attribute twice is harmless)
        if (!lds_set.load(std::memory_order_acquire)) {
            ST_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&st::value_model_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)st::vm_lds_bytes(st::kVmDepth)));
            lds_set.store(true, std::memory_order_release);
        }
        TimedLaunch t(0, (hipStream_t)hip_stream);
        hipLaunchKernelGGL(st::value_model_kernel, dim3(grid), dim3(st::kVmThreads),
                           st::vm_lds_bytes(deepest), (hipStream_t)hip_stream,
                           dev_task_scores, n, n_tasks, prog, st::vm_lds_slots(deepest), dev_out);
    }
    ST_HIP(hipGetLastError());
    return ST_OK;
}

int st_score_pairs(const int8_t* dev_items, const float* dev_item_scale, int32_t d, const int8_t* dev_queries,
                   const float* dev_query_scale, const int64_t* dev_pair_item, const int32_t* dev_pair_query,
                   int64_t n_pairs, int32_t* dev_out_dot, float* dev_out_score, void* hip_stream)
{
    if (!dev_items || !dev_item_scale || !dev_queries || !dev_query_scale || !dev_pair_item || !dev_pair_query)
        return fail(ST_EINVAL, "null argument");
    if (d < 16 || d > ST_MAX_DIM || d % 16) return fail(ST_EINVAL, "d=%d must be a multiple of 16", d);
    if (n_pairs < 0) return fail(ST_EINVAL, "n_pairs negative");
    if (n_pairs == 0) return ST_OK;
    const unsigned grid = (unsigned)((n_pairs + 255) / 256);
    hipLaunchKernelGGL(st::score_pairs_kernel, dim3(grid), dim3(256), 0, (hipStream_t)hip_stream, dev_items,
                       dev_item_scale, d, dev_queries, dev_query_scale, dev_pair_item, dev_pair_query, n_pairs,
                       dev_out_dot, dev_out_score);
    ST_HIP(hipGetLastError());
    return ST_OK;
}

}  // extern "C"
