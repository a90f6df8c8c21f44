// C ABI of the library (declared in tdfa.h): handles, argument checks, host-side vocabulary
// packing, and kernel launches.  Every table entry, mask and token choice is computed by the
// kernels; the host packs the vocabulary and prepares an automaton for them (plan.hip).
#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <cstdint>
#include <memory>
#include <mutex>
#include <new>
#include <vector>

#include "tdfa_internal.h"

struct tdfa_vocab {
    int32_t n_tokens = 0;
    int64_t n_bytes = 0;
    int32_t max_len = 0;
    uint32_t* words = nullptr;   // device: token bytes, each token padded to a multiple of 4 bytes
    uint32_t* off = nullptr;     // device [n_tokens + 1]: word offset of each token
    uint32_t* len = nullptr;     // device [n_tokens]: byte length
    uint8_t* sorted = nullptr;   // device [n_tokens]: blocked trie order (see tdfa_vocab_create)
    uint32_t* prefix = nullptr;  // device [n_tokens][8]: the first 32 bytes of each token, zero padded
    // for the sweep (sweep.hip): tokens with a third / fourth byte grouped by that byte, in chunks of at
    // most kSweepChunk tokens of one byte; tokens of five or more bytes
    int32_t* group_tokens[2] = {nullptr, nullptr};
    int32_t* group_chunks[2] = {nullptr, nullptr};
    int32_t n_group_chunks[2] = {0, 0};
    int32_t* tail_tokens = nullptr;
    int32_t n_tail = 0;
};

namespace tdfa {
// An event recorded on a stream behind the last launches that read or wrote an automaton's device memory.
struct UseEvent {
    hipEvent_t ev = nullptr;
    ~UseEvent()
    {
        if (ev) (void)hipEventDestroy(ev);
    }
};
}  // namespace tdfa

struct tdfa_dfa {
    int32_t n_states = 0;
    int32_t start = 0;
    int32_t q_stride = 0;
    bool narrow = false;
    int32_t* trans = nullptr;    // device [n_states][256]
    uint8_t* accept = nullptr;   // device [n_states]
    void* trans_t = nullptr;     // device workspace for the transposed table
    int32_t* order = nullptr;    // device [n_order]: the states in the order the compile kernel's lanes take them
    unsigned char* plan = nullptr;   // device: clean sets, group classes, jump tables (layout in tdfa_internal.h)
    int32_t n_order = 0;
    bool has_jump = false;
    // workspace of a compile call (written by its first kernel, read by the second): one byte per
    // (64-state group, token); sized for the vocabulary of the latest call
    mutable uint8_t* start_bytes = nullptr;
    mutable size_t start_cap = 0;
    size_t start_limit = (size_t)1 << 30;   // largest such workspace (tdfa_dfa_workspace_limit)
    // the level-by-level sweep (sweep.hip): workspace allocated and sized by the first compile call
    // that takes that path (and again for a vocabulary that needs more)
    int64_t n_pairs = 0;
    int path = TDFA_PATH_AUTO;
    mutable tdfa::SweepWorkspace sweep;
    mutable bool sweep_too_large = false;
    // the blocks above that came from the cache of automaton memory (pointer, bytes), the last launches
    // that used them, and whether a launch under stream capture did (no event can tell when that ends)
    mutable std::vector<std::pair<void*, size_t>> cached;
    mutable std::shared_ptr<tdfa::UseEvent> used;
    mutable hipStream_t used_stream = nullptr;
    mutable bool used_in_capture = false;
};

struct tdfa_table {
    int64_t n_rows = 0;
    int32_t n_tokens = 0;
    int64_t row_words = 0;
    int32_t* delta = nullptr;           // dense rows; NULL in a packed table
    uint32_t* allow = nullptr;
    bool own_delta = false, own_allow = false;
    uint32_t* row_allowed = nullptr;    // device [n_rows] from the pool, or NULL: tokens each state allows (tables the library wrote)
    // packed form (tdfa_table_pack), owned by the table
    int32_t* targets = nullptr;
    int64_t* row_begin = nullptr;
    uint32_t* dir = nullptr;
    int64_t n_edges = 0;
};

namespace tdfa {

static thread_local char g_error[512] = "";

int fail(int code, const char* fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_error, sizeof(g_error), fmt, ap);
    va_end(ap);
    return code;
}

void clear_error() { g_error[0] = '\0'; }

void vocab_view(const tdfa_vocab* vocab, VocabView* out)
{
    out->words = vocab->words;
    out->off = vocab->off;
    out->len = vocab->len;
    out->n_tokens = vocab->n_tokens;
}

namespace {

void cache_trim();

// hipMalloc; if the device is out of memory, once more after the library's cached blocks have gone back to it.
int device_malloc(void** p, size_t bytes)
{
    *p = nullptr;
    hipError_t e = hipMalloc(p, bytes ? bytes : 1);
    if (e == hipErrorOutOfMemory) {
        (void)hipGetLastError();
        cache_trim();
        e = hipMalloc(p, bytes ? bytes : 1);
    }
    if (e != hipSuccess) {
        *p = nullptr;
        return fail(e == hipErrorOutOfMemory ? TDFA_E_OOM : TDFA_E_DEVICE, "hipMalloc of %zu bytes: %s", bytes, hipGetErrorString(e));
    }
    return TDFA_OK;
}

template <typename T>
int device_alloc(T** p, size_t count)
{
    void* v = nullptr;
    const int rc = device_malloc(&v, (count ? count : 1) * sizeof(T));
    *p = static_cast<T*>(v);
    return rc;
}

int static_scratch(void** out);

// Device memory of automaton handles is kept for the next handle instead of going back to the runtime:
// hipFree waits for all work on the device, and a caller that prepares its next constraint while the GPU
// still decodes under the last one would stall on every destroyed automaton.  A block carries the event
// recorded behind the last launches that used it and is handed out again only when that has completed.
struct CachedBlock {
    void* ptr;
    size_t bytes;
    int device;
    std::shared_ptr<UseEvent> used;
};
std::mutex g_cache_mutex;
std::vector<CachedBlock> g_cache;              // free blocks, oldest first
size_t g_cache_bytes = 0;
constexpr size_t kCacheMaxBytes = (size_t)4 << 30, kCacheMaxBlocks = 256;

bool use_completed(const std::shared_ptr<UseEvent>& used)
{
    if (!used || !used->ev) return true;
    const hipError_t e = hipEventQuery(used->ev);
    if (e != hipSuccess) (void)hipGetLastError();      // "not ready" is no error of ours
    return e == hipSuccess;
}

int cache_alloc(void** out, size_t bytes)
{
    *out = nullptr;
    if (!bytes) bytes = 1;
    int dev = 0;
    TDFA_HIP(hipGetDevice(&dev));
    std::shared_ptr<UseEvent> wait_for;
    {
        std::lock_guard<std::mutex> lock(g_cache_mutex);
        size_t busy = g_cache.size();
        for (size_t i = 0; i < g_cache.size(); ++i) {
            CachedBlock& b = g_cache[i];
            if (b.device != dev || b.bytes < bytes || b.bytes > 2 * bytes + ((size_t)64 << 10)) continue;
            if (use_completed(b.used)) {
                *out = b.ptr;
                g_cache_bytes -= b.bytes;
                g_cache.erase(g_cache.begin() + (long)i);
                return TDFA_OK;
            }
            if (busy == g_cache.size()) busy = i;
        }
        // every fitting block is still in use: a new one while the cache is small, else wait for the oldest
        if (busy != g_cache.size() && g_cache_bytes > kCacheMaxBytes / 2) {
            *out = g_cache[busy].ptr;
            wait_for = g_cache[busy].used;
            g_cache_bytes -= g_cache[busy].bytes;
            g_cache.erase(g_cache.begin() + (long)busy);
        }
    }
    if (*out) {
        TDFA_HIP(hipEventSynchronize(wait_for->ev));
        return TDFA_OK;
    }
    return device_malloc(out, bytes);
}

// The block goes to the cache; `used` (may be empty) tells when the GPU is done with it.
void cache_free(void* p, size_t bytes, const std::shared_ptr<UseEvent>& used)
{
    if (!p) return;
    int dev = 0;
    (void)hipGetDevice(&dev);
    std::vector<void*> to_free;
    {
        std::lock_guard<std::mutex> lock(g_cache_mutex);
        g_cache.push_back(CachedBlock{p, bytes, dev, used});
        g_cache_bytes += bytes;
        while (g_cache.size() > kCacheMaxBlocks || g_cache_bytes > kCacheMaxBytes) {
            to_free.push_back(g_cache.front().ptr);
            g_cache_bytes -= g_cache.front().bytes;
            g_cache.erase(g_cache.begin());
        }
    }
    for (void* q : to_free) (void)hipFree(q);          // (waits for the device: whatever used the block is done)
}

void cache_trim()
{
    std::vector<void*> to_free;
    {
        std::lock_guard<std::mutex> lock(g_cache_mutex);
        for (const CachedBlock& b : g_cache) to_free.push_back(b.ptr);
        g_cache.clear();
        g_cache_bytes = 0;
    }
    for (void* q : to_free) (void)hipFree(q);
}

// A block of an automaton handle from the cache, remembered in the handle.
template <typename T>
int dfa_alloc(const tdfa_dfa* d, T** p, size_t count)
{
    void* v = nullptr;
    const size_t bytes = (count ? count : 1) * sizeof(T);
    const int rc = cache_alloc(&v, bytes);
    *p = static_cast<T*>(v);
    if (rc == TDFA_OK) d->cached.emplace_back(v, bytes);
    return rc;
}

// One stream per device for the uploads of tdfa_dfa_create, so that creating an automaton waits for its own
// copies only and not for whatever the caller's stream still holds.
int upload_stream(hipStream_t* out)
{
    static std::mutex m;
    constexpr int kStreams = 64;
    static hipStream_t streams[kStreams] = {};
    int dev = 0;
    TDFA_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kStreams) return fail(TDFA_E_UNSUPPORTED, "device index %d", dev);
    std::lock_guard<std::mutex> lock(m);
    if (!streams[dev]) TDFA_HIP(hipStreamCreateWithFlags(&streams[dev], hipStreamNonBlocking));
    *out = streams[dev];
    return TDFA_OK;
}

// Before the launches of a compile call on stream s: an automaton last used on another stream is waited for there.
int before_use(const tdfa_dfa* d, hipStream_t s)
{
    if (d->used && d->used->ev && d->used_stream != s) TDFA_HIP(hipStreamWaitEvent(s, d->used->ev, 0));
    return TDFA_OK;
}

// Behind the launches of a compile call on stream s: one event for all its automata.
int after_use(const tdfa_dfa* const* dfas, int32_t n, hipStream_t s)
{
    hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
    TDFA_HIP(hipStreamIsCapturing(s, &cs));
    if (cs != hipStreamCaptureStatusNone) {
        for (int32_t i = 0; i < n; ++i) dfas[i]->used_in_capture = true;
        return TDFA_OK;
    }
    std::shared_ptr<UseEvent> ev;
    try {
        ev = std::make_shared<UseEvent>();
    } catch (const std::bad_alloc&) {
        return fail(TDFA_E_OOM, "host allocation failed");
    }
    TDFA_HIP(hipEventCreateWithFlags(&ev->ev, hipEventDisableTiming));
    TDFA_HIP(hipEventRecord(ev->ev, s));
    for (int32_t i = 0; i < n; ++i) {
        dfas[i]->used = ev;
        dfas[i]->used_stream = s;
    }
    return TDFA_OK;
}

int make_table(int64_t n_rows, int32_t n_tokens, int32_t* delta_dev, uint32_t* allow_dev, tdfa_table** out)
{
    tdfa_table* t = new (std::nothrow) tdfa_table;
    if (!t) return fail(TDFA_E_OOM, "host allocation failed");
    t->n_rows = n_rows;
    t->n_tokens = n_tokens;
    t->row_words = allow_row_words(n_tokens);
    t->delta = delta_dev;
    t->allow = allow_dev;
    int rc = TDFA_OK;
    if (!t->delta) {
        rc = device_alloc(&t->delta, (size_t)n_rows * (size_t)n_tokens);
        t->own_delta = rc == TDFA_OK;
    }
    if (rc == TDFA_OK && !t->allow) {
        rc = device_alloc(&t->allow, (size_t)n_rows * (size_t)t->row_words);
        t->own_allow = rc == TDFA_OK;
    }
    if (rc != TDFA_OK) {
        if (t->own_delta) (void)hipFree(t->delta);
        delete t;
        return rc;
    }
    {
        // every table passes here before its first decode step: the address of the static scratch is
        // then already known when a step that must not call into the runtime's set-up paths needs it
        void* unused = nullptr;
        if (static_scratch(&unused) != TDFA_OK) clear_error();
    }
    *out = t;
    return TDFA_OK;
}

// The tokens every row of `t` allows, counted by a kernel after the library has written (or edited) the
// table's allowed bits.  Tables over buffers that the caller filled (tdfa_table_wrap) have no counts.
int count_rows(tdfa_table* t, hipStream_t s);

// Cross-workgroup reduction scratch of the decode step: one per device, shared by every table
// on it, all zero between launches.  A block that has been handed to a launch is never freed
// (a recorded graph may still name it): growing allocates a larger block and keeps the old one
// until the process ends.
struct DeviceScratch {
    unsigned long long* best = nullptr;
    unsigned int* count = nullptr;      // [2 * cap]: arrival counters, then scratch words that need not be zero
    int32_t cap = 0;
};
constexpr int kMaxDevices = 64;
DeviceScratch g_scratch[kMaxDevices];
std::mutex g_scratch_mutex;

int ensure_scratch(int32_t batch, hipStream_t stream, DeviceScratch* out)
{
    int dev = 0;
    TDFA_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return fail(TDFA_E_UNSUPPORTED, "device index %d", dev);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    DeviceScratch* sc = &g_scratch[dev];
    if (batch <= sc->cap) {
        *out = *sc;
        return TDFA_OK;
    }
    // Growing allocates and clears, which a stream capture must not contain.
    hipStreamCaptureStatus capturing = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(stream, &capturing) != hipSuccess) (void)hipGetLastError();
    if (capturing != hipStreamCaptureStatusNone)
        return fail(TDFA_E_UNSUPPORTED,
                    "the reduction scratch must grow for batch %d, which cannot happen inside a stream capture: "
                    "make one step at this batch size before capturing",
                    batch);
    int32_t cap = sc->cap ? sc->cap : 4096;
    while (cap < batch) cap *= 2;
    DeviceScratch grown;
    int rc = device_alloc(&grown.best, (size_t)cap);
    if (rc != TDFA_OK) return rc;
    rc = device_alloc(&grown.count, 2 * (size_t)cap);      // second half: the top-k cuts of a sampling step
    if (rc != TDFA_OK) {
        (void)hipFree(grown.best);
        return rc;
    }
    // cleared before the call returns, so a step on any stream finds zeros
    TDFA_HIP(hipMemset(grown.best, 0, sizeof(unsigned long long) * (size_t)cap));
    TDFA_HIP(hipMemset(grown.count, 0, sizeof(unsigned int) * 2 * (size_t)cap));
    grown.cap = cap;
    *sc = grown;                                             // the old block, if any, stays allocated
    *out = grown;
    return TDFA_OK;
}

// The same scratch for callers that cannot allocate (tdfa_mask_step_noalloc): a fixed array in the
// library's device image.  Each GPU holds its own copy at its own address; the name below is only
// a handle for hipGetSymbolAddress, host code uses the per-device pointer it returns.
constexpr int32_t kStaticMaxBatch = 4096;
constexpr size_t kStaticScratchBytes = (size_t)kStaticMaxBatch * (sizeof(unsigned long long) + sizeof(unsigned int));
}  // namespace

int step_scratch(int32_t batch, hipStream_t stream, unsigned long long** best, unsigned int** count)
{
    DeviceScratch sc;
    const int rc = ensure_scratch(batch, stream, &sc);
    if (rc != TDFA_OK) return rc;
    *best = sc.best;
    *count = sc.count;
    return TDFA_OK;
}
}  // namespace tdfa
static __device__ __align__(256) unsigned char scratch[tdfa::kStaticScratchBytes];
namespace tdfa {
namespace {
void* g_static_ptr[kMaxDevices];
std::mutex g_static_mutex;

// The device address of `scratch` on the current device (looked up once per device).
int static_scratch(void** out)
{
    int dev = 0;
    TDFA_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return fail(TDFA_E_UNSUPPORTED, "device index %d", dev);
    std::lock_guard<std::mutex> lock(g_static_mutex);
    if (!g_static_ptr[dev]) {
        void* ptr = nullptr;
        const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr)
            return fail(TDFA_E_DEVICE, "hipGetSymbolAddress(scratch): %s", hipGetErrorString(e));
        g_static_ptr[dev] = ptr;
    }
    *out = g_static_ptr[dev];
    return TDFA_OK;
}

constexpr int32_t kPairsMinStates = 8192;   // smaller automata: their transposed table sits in the caches, the walk is fine

bool takes_pairs(const tdfa_dfa* d)
{
    const bool possible = d->narrow && !d->has_jump && d->n_pairs > 0 && !d->sweep_too_large;
    if (d->path == TDFA_PATH_PAIRS) return possible;
    if (d->path == TDFA_PATH_AUTO) return possible && d->n_states >= kPairsMinStates;
    return false;
}

// The sweep's four large arrays (two lists, two buffers: gigabytes for an automaton like c4's) come
// from a small pool: a destroyed automaton's blocks are kept for the next one instead of going back
// to the driver, whose allocation calls cost as much as a tenth of such a compile.  At most
// kPoolBlocks blocks are kept per process (the oldest is freed first); tdfa_trim() frees them all.
constexpr size_t kPoolBlocks = 8;
struct PoolBlock {
    void* ptr;
    size_t bytes;
    int device;
};
std::mutex g_pool_mutex;
std::vector<PoolBlock> g_pool;                 // free blocks, oldest first
std::vector<PoolBlock> g_pool_taken;           // blocks in use (their true sizes)

int pool_alloc(uint32_t** out, size_t count)
{
    *out = nullptr;
    const size_t bytes = (count ? count : 1) * sizeof(uint32_t);
    int dev = 0;
    TDFA_HIP(hipGetDevice(&dev));
    {
        std::lock_guard<std::mutex> lock(g_pool_mutex);
        size_t best = g_pool.size();
        for (size_t i = 0; i < g_pool.size(); ++i)
            if (g_pool[i].device == dev && g_pool[i].bytes >= bytes && g_pool[i].bytes <= 2 * bytes + ((size_t)1 << 20) &&
                (best == g_pool.size() || g_pool[i].bytes < g_pool[best].bytes))
                best = i;
        if (best != g_pool.size()) {
            g_pool_taken.push_back(g_pool[best]);
            *out = static_cast<uint32_t*>(g_pool[best].ptr);
            g_pool.erase(g_pool.begin() + (long)best);
            return TDFA_OK;
        }
    }
    void* p = nullptr;
    TDFA_HIP(hipMalloc(&p, bytes));
    std::lock_guard<std::mutex> lock(g_pool_mutex);
    g_pool_taken.push_back(PoolBlock{p, bytes, dev});
    *out = static_cast<uint32_t*>(p);
    return TDFA_OK;
}

// The caller has made sure that no kernel still uses the block.
void pool_release(void* p)
{
    if (!p) return;
    std::vector<void*> to_free;
    {
        std::lock_guard<std::mutex> lock(g_pool_mutex);
        for (size_t i = 0; i < g_pool_taken.size(); ++i)
            if (g_pool_taken[i].ptr == p) {
                g_pool.push_back(g_pool_taken[i]);
                g_pool_taken.erase(g_pool_taken.begin() + (long)i);
                break;
            }
        while (g_pool.size() > kPoolBlocks) {
            to_free.push_back(g_pool.front().ptr);
            g_pool.erase(g_pool.begin());
        }
    }
    for (void* q : to_free) (void)hipFree(q);
}

int count_rows(tdfa_table* t, hipStream_t s)
{
    if (t->n_rows <= 0) return TDFA_OK;
    if (!t->row_allowed) {
        const int rc = pool_alloc(&t->row_allowed, (size_t)t->n_rows);
        if (rc != TDFA_OK) return rc;
    }
    return launch_row_allowed(t->allow, t->n_rows, t->n_tokens, t->row_words, t->row_allowed, s);
}

void free_sweep(SweepWorkspace* ws)
{
    for (uint32_t* p : {ws->n1, ws->off1, ws->cnt2, ws->err, ws->need, ws->cnt3, ws->cntF})
        if (p) (void)hipFree(p);
    if (ws->chunk_sum) (void)hipFree(ws->chunk_sum);
    if (ws->list1 || ws->list2 || ws->buf_a || ws->buf_b) {
        (void)hipDeviceSynchronize();              // (the frees above wait too when there are any; this covers the rest)
        for (uint32_t* p : {ws->list1, ws->list2, ws->buf_a, ws->buf_b}) pool_release(p);
    }
    *ws = SweepWorkspace();
}

CompileArgs args_of(const tdfa_vocab* v, const tdfa_table* t, const CompileEntry* entries, int32_t n);

// The sweep's workspace for automaton d and vocabulary v: allocated on first use and sized from what
// the first kernels of the sweep report (the lists of level 2 depend on the automaton, the two
// buffers of the later levels on the vocabulary as well), which takes two waits for the device; later
// calls with the same vocabulary find everything in place.  *usable = false: it would exceed eight
// times the automaton's workspace limit, compile by the walk instead.
int prepare_sweep(const tdfa_dfa* d, const tdfa_vocab* v, CompileEntry* e, hipStream_t s, bool* usable)
{
    SweepWorkspace& ws = d->sweep;
    *usable = true;
    int rc = TDFA_OK;
    if (!ws.n1) {
        rc = device_alloc(&ws.n1, 256);
        if (rc == TDFA_OK) rc = device_alloc(&ws.off1, 257);
        if (rc == TDFA_OK) rc = device_alloc(&ws.cnt2, 65536);
        if (rc == TDFA_OK) rc = device_alloc(&ws.err, 1);
        if (rc != TDFA_OK) return rc;
    }
    if (ws.token_cap < v->n_tokens || !ws.need) {
        TDFA_HIP(hipStreamSynchronize(s));                      // an earlier launch may still use the old arrays
        for (uint32_t** p : {&ws.need, &ws.cnt3, &ws.cntF}) {
            if (*p) (void)hipFree(*p);
            *p = nullptr;
        }
        if (ws.chunk_sum) (void)hipFree(ws.chunk_sum);
        ws.chunk_sum = nullptr;
        rc = device_alloc(&ws.chunk_sum, (size_t)v->n_tokens / 1024 + 2);
        if (rc == TDFA_OK) rc = device_alloc(&ws.need, (size_t)v->n_tokens + 1);
        if (rc == TDFA_OK) rc = device_alloc(&ws.cnt3, (size_t)v->n_tokens);
        if (rc == TDFA_OK) rc = device_alloc(&ws.cntF, (size_t)v->n_tokens);
        if (rc != TDFA_OK) return rc;
        ws.token_cap = v->n_tokens;
        ws.buffers_sized = false;
    }
    e->use_pairs = true;
    e->sweep = &ws;
    e->start_bytes = nullptr;
    e->has_jump = false;
    const size_t limit = d->start_limit > ((size_t)1 << 60) ? d->start_limit : d->start_limit * 8;
    const CompileArgs a = args_of(v, nullptr, e, 1);
    if (!ws.sized) {
        rc = launch_compile_sweep(a, *e, s);
        if (rc != TDFA_OK) return rc;
        uint32_t total1 = 0;
        TDFA_HIP(hipMemcpyAsync(&total1, ws.off1 + 256, sizeof(uint32_t), hipMemcpyDeviceToHost, s));
        TDFA_HIP(hipStreamSynchronize(s));
        const uint64_t cap = (uint64_t)256 * total1;
        if (cap * 4 > limit || cap >= 0xFFFFFFFFull) {
            d->sweep_too_large = true;
            *usable = false;
            return TDFA_OK;
        }
        rc = pool_alloc(&ws.list2, (size_t)cap);
        if (rc == TDFA_OK) rc = pool_alloc(&ws.list1, (size_t)total1);
        if (rc != TDFA_OK) return rc;
        ws.list2_cap = cap;
        ws.sized = true;
    }
    if (!ws.buffers_sized || ws.sized_for != v) {
        ws.buffers_sized = false;
        rc = launch_compile_sweep(a, *e, s);
        if (rc != TDFA_OK) return rc;
        unsigned long long total = 0;
        TDFA_HIP(hipMemcpyAsync(&total, ws.chunk_sum + (v->n_tokens / 1024 + 1), sizeof(total), hipMemcpyDeviceToHost, s));
        TDFA_HIP(hipStreamSynchronize(s));
        if (total >= 0xFFFFFFFFull || (ws.list2_cap + 2 * (uint64_t)total) * 4 > limit) {
            d->sweep_too_large = true;
            *usable = false;
            return TDFA_OK;
        }
        if ((uint64_t)total > ws.buf_cap) {
            if (ws.buf_a || ws.buf_b) {
                TDFA_HIP(hipDeviceSynchronize());   // an earlier launch may still use them
                pool_release(ws.buf_a);
                pool_release(ws.buf_b);
            }
            ws.buf_a = ws.buf_b = nullptr;
            ws.buf_cap = 0;
            rc = pool_alloc(&ws.buf_a, (size_t)total);
            if (rc == TDFA_OK) rc = pool_alloc(&ws.buf_b, (size_t)total);
            if (rc != TDFA_OK) return rc;
            ws.buf_cap = total;
        }
        ws.buffers_sized = true;
        ws.sized_for = v;
        ws.lists_ready = true;              // the caller's compile launch comes next on this stream
    }
    return TDFA_OK;
}

int entry_of(const tdfa_dfa* d, const tdfa_vocab* vocab, int32_t out_row, int32_t state_base, hipStream_t stream, CompileEntry* out)
{
    const int32_t n_tokens = vocab->n_tokens;
    CompileEntry e;
    e.trans = d->trans;
    e.trans_t = d->trans_t;
    e.order = d->order;
    e.plan = d->plan;
    e.n_order = d->n_order;
    e.narrow = d->narrow;
    e.n_states = d->n_states;
    e.q_stride = d->q_stride;
    e.out_row = out_row;
    e.state_base = state_base;
    e.use_pairs = false;
    e.sweep = nullptr;
    e.staged = d->path == TDFA_PATH_STAGED && d->narrow && (size_t)256 * d->q_stride * 2 <= tdfa::kStagedTableBytes;
    e.start_bytes = nullptr;
    e.has_jump = false;
    // Which kernels compile this automaton.  The sweep pays where the byte-by-byte walk is at its worst:
    // a large automaton (its transposed table does not stay in a compute unit's caches) with no
    // counter-like class to jump over.
    if (n_tokens > 0 && takes_pairs(d)) {
        bool usable = false;
        const int rc = prepare_sweep(d, vocab, &e, stream, &usable);
        if (rc != TDFA_OK) return rc;
        if (usable) {
            *out = e;
            return TDFA_OK;
        }
        e.use_pairs = false;
        e.sweep = nullptr;
    }
    const size_t need = (size_t)((d->n_order + 63) / 64) * (size_t)(n_tokens > 0 ? n_tokens : 0);
    // An automaton that would need more than its limit is compiled without start bytes (every
    // group looks up every token's first byte, no jump tables).
    if (need > d->start_limit) {
        e.start_bytes = nullptr;
        e.has_jump = false;
    } else {
        if (need > d->start_cap) {
            // the old, smaller buffer stays with the handle (an earlier launch may still read it) until the handle goes
            d->start_bytes = nullptr;
            d->start_cap = 0;
            const int rc = dfa_alloc(d, &d->start_bytes, need);
            if (rc != TDFA_OK) return rc;
            d->start_cap = need;
        }
        e.start_bytes = d->start_bytes;
        e.has_jump = d->has_jump;
    }
    *out = e;
    return TDFA_OK;
}

CompileArgs args_of(const tdfa_vocab* v, const tdfa_table* t, const CompileEntry* entries, int32_t n)
{
    CompileArgs a;
    a.entries = entries;
    a.n = n;
    a.vwords = v->words;
    a.voff = v->off;
    a.vlen = v->len;
    a.vsorted = v->sorted;
    a.vprefix = v->prefix;
    a.n_tokens = v->n_tokens;
    for (int i = 0; i < 2; ++i) {
        a.group_tokens[i] = v->group_tokens[i];
        a.group_chunks[i] = v->group_chunks[i];
        a.n_group_chunks[i] = v->n_group_chunks[i];
    }
    a.tail_tokens = v->tail_tokens;
    a.n_tail = v->n_tail;
    a.delta = t ? t->delta : nullptr;
    a.allow = t ? t->allow : nullptr;
    a.row_words = t ? t->row_words : 0;
    return a;
}

}  // namespace
}  // namespace tdfa

using namespace tdfa;

extern "C" {

const char* tdfa_last_error(void) { return g_error; }

int tdfa_version(void) { return 100; }

int64_t tdfa_allow_row_words(int32_t n_tokens) { return allow_row_words(n_tokens); }

int tdfa_vocab_create(const uint8_t* bytes, const uint64_t* offsets, int32_t n_tokens, void* stream,
                      tdfa_vocab** out)
{
    clear_error();
    if (!out) return fail(TDFA_E_INVALID_ARG, "out is NULL");
    *out = nullptr;
    if (!offsets) return fail(TDFA_E_INVALID_ARG, "offsets is NULL");
    if (n_tokens < 0 || n_tokens > (1 << 24)) return fail(TDFA_E_INVALID_ARG, "n_tokens %d outside [0, 2^24]", n_tokens);
    uint64_t n_words = 0;
    int64_t max_len = 0;
    for (int32_t t = 0; t < n_tokens; ++t) {
        if (offsets[t + 1] < offsets[t]) return fail(TDFA_E_INVALID_ARG, "offsets decrease at token %d", t);
        const uint64_t len = offsets[t + 1] - offsets[t];
        if (len > 0x7FFFFFFFull) return fail(TDFA_E_INVALID_ARG, "token %d is longer than 2^31 bytes", t);
        n_words += (len + 3) / 4;
        if ((int64_t)len > max_len) max_len = (int64_t)len;
    }
    const uint64_t n_bytes = n_tokens ? offsets[n_tokens] - offsets[0] : 0;
    if (n_bytes > 0 && !bytes) return fail(TDFA_E_INVALID_ARG, "bytes is NULL");
    if (n_words >= 0xFFFFFFFFull) return fail(TDFA_E_UNSUPPORTED, "vocabulary holds more than 16 GiB of bytes");

    std::vector<uint32_t> words, off, len, prefix;
    try {
        prefix.assign(((size_t)n_tokens + 1) * 8, 0u);
        words.assign((size_t)n_words + 1, 0u);
        off.resize((size_t)n_tokens + 1);
        len.resize((size_t)n_tokens + 1);
    } catch (const std::bad_alloc&) {
        return fail(TDFA_E_OOM, "host allocation failed");
    }
    uint64_t w = 0;
    for (int32_t t = 0; t < n_tokens; ++t) {
        const uint64_t n = offsets[t + 1] - offsets[t];
        off[t] = (uint32_t)w;
        len[t] = (uint32_t)n;
        if (n) std::memcpy(reinterpret_cast<uint8_t*>(words.data()) + w * 4, bytes + offsets[t], (size_t)n);
        if (n) std::memcpy(prefix.data() + (size_t)t * 8, bytes + offsets[t], (size_t)std::min<uint64_t>(n, 32));
        w += (n + 3) / 4;
    }
    off[n_tokens] = (uint32_t)w;
    len[n_tokens] = 0;

    // Blocked prefix-trie order: inside every block of kVocabSortBlock consecutive ids the tokens
    // are listed in byte-lexicographic order, so tokens that share a prefix are neighbours (the
    // compact T_V merges exactly those prefixes).  Columns of the table stay in id order; only
    // the order in which a tile's tokens are walked changes.
    std::vector<uint8_t> sorted;
    try {
        sorted.resize((size_t)n_tokens + 1);
    } catch (const std::bad_alloc&) {
        return fail(TDFA_E_OOM, "host allocation failed");
    }
    for (int32_t b0 = 0; b0 < n_tokens; b0 += kVocabSortBlock) {
        const int32_t n = std::min<int32_t>(kVocabSortBlock, n_tokens - b0);
        uint8_t* idx = sorted.data() + b0;
        for (int32_t i = 0; i < n; ++i) idx[i] = (uint8_t)i;
        if (!bytes) continue;                            // every token is empty
        std::sort(idx, idx + n, [&](uint8_t x, uint8_t y) {
            const uint64_t lx = offsets[b0 + x + 1] - offsets[b0 + x], ly = offsets[b0 + y + 1] - offsets[b0 + y];
            const int c = std::memcmp(bytes + offsets[b0 + x], bytes + offsets[b0 + y], (size_t)std::min(lx, ly));
            if (c != 0) return c < 0;
            if (lx != ly) return lx < ly;
            return x < y;
        });
    }

    // For the sweep over prefix lists (sweep.hip): the tokens that have a third byte grouped by that
    // byte, likewise for the fourth, each group cut into chunks of at most kSweepChunk tokens (one
    // workgroup each); and the tokens of five or more bytes.
    constexpr int kSweepChunk = 16;
    std::vector<int32_t> group_tokens[2], group_chunks[2], tail_tokens;
    try {
        for (int lvl = 0; lvl < 2; ++lvl) {
            const uint64_t at = 2 + (uint64_t)lvl;                  // index of the byte that groups
            std::vector<int32_t> count(257, 0);
            for (int32_t t = 0; t < n_tokens; ++t)
                if (offsets[t + 1] - offsets[t] > at) ++count[(size_t)bytes[offsets[t] + at] + 1];
            for (int b = 0; b < 256; ++b) count[(size_t)b + 1] += count[(size_t)b];
            group_tokens[lvl].resize((size_t)count[256] + 1);
            std::vector<int32_t> fill(count.begin(), count.end() - 1);
            for (int32_t t = 0; t < n_tokens; ++t)
                if (offsets[t + 1] - offsets[t] > at) group_tokens[lvl][(size_t)fill[bytes[offsets[t] + at]]++] = t;
            for (int b = 0; b < 256; ++b)
                for (int32_t first = count[(size_t)b]; first < count[(size_t)b + 1]; first += kSweepChunk) {
                    group_chunks[lvl].push_back(b);
                    group_chunks[lvl].push_back(first);
                    group_chunks[lvl].push_back(std::min<int32_t>(kSweepChunk, count[(size_t)b + 1] - first));
                }
            group_chunks[lvl].push_back(0);                         // never empty
        }
        for (int32_t t = 0; t < n_tokens; ++t)
            if (offsets[t + 1] - offsets[t] >= 5) tail_tokens.push_back(t);
        tail_tokens.push_back(0);
    } catch (const std::bad_alloc&) {
        return fail(TDFA_E_OOM, "host allocation failed");
    }

    tdfa_vocab* v = new (std::nothrow) tdfa_vocab;
    if (!v) return fail(TDFA_E_OOM, "host allocation failed");
    v->n_tokens = n_tokens;
    for (int lvl = 0; lvl < 2; ++lvl) v->n_group_chunks[lvl] = (int32_t)(group_chunks[lvl].size() / 3);
    v->n_tail = (int32_t)tail_tokens.size() - 1;
    v->n_bytes = (int64_t)n_bytes;
    v->max_len = (int32_t)max_len;
    hipStream_t s = static_cast<hipStream_t>(stream);
    int rc = device_alloc(&v->words, words.size());
    if (rc == TDFA_OK) rc = device_alloc(&v->off, off.size());
    if (rc == TDFA_OK) rc = device_alloc(&v->len, len.size());
    if (rc == TDFA_OK) rc = device_alloc(&v->sorted, sorted.size());
    if (rc == TDFA_OK) rc = device_alloc(&v->prefix, prefix.size());
    for (int lvl = 0; lvl < 2; ++lvl) {
        if (rc == TDFA_OK) rc = device_alloc(&v->group_tokens[lvl], group_tokens[lvl].size());
        if (rc == TDFA_OK) rc = device_alloc(&v->group_chunks[lvl], group_chunks[lvl].size());
    }
    if (rc == TDFA_OK) rc = device_alloc(&v->tail_tokens, tail_tokens.size());
    auto copy = [&](void* dst, const void* src, size_t n) -> int {
        TDFA_HIP(hipMemcpyAsync(dst, src, n, hipMemcpyHostToDevice, s));
        return TDFA_OK;
    };
    if (rc == TDFA_OK) rc = copy(v->words, words.data(), words.size() * 4);
    if (rc == TDFA_OK) rc = copy(v->off, off.data(), off.size() * 4);
    if (rc == TDFA_OK) rc = copy(v->len, len.data(), len.size() * 4);
    if (rc == TDFA_OK) rc = copy(v->sorted, sorted.data(), sorted.size());
    if (rc == TDFA_OK) rc = copy(v->prefix, prefix.data(), prefix.size() * 4);
    for (int lvl = 0; lvl < 2; ++lvl) {
        if (rc == TDFA_OK) rc = copy(v->group_tokens[lvl], group_tokens[lvl].data(), group_tokens[lvl].size() * 4);
        if (rc == TDFA_OK) rc = copy(v->group_chunks[lvl], group_chunks[lvl].data(), group_chunks[lvl].size() * 4);
    }
    if (rc == TDFA_OK) rc = copy(v->tail_tokens, tail_tokens.data(), tail_tokens.size() * 4);
    if (rc == TDFA_OK) {
        hipError_t e = hipStreamSynchronize(s);
        if (e != hipSuccess) rc = fail(TDFA_E_DEVICE, "hipStreamSynchronize: %s", hipGetErrorString(e));
    }
    if (rc != TDFA_OK) {
        tdfa_vocab_destroy(v);
        return rc;
    }
    *out = v;
    return TDFA_OK;
}

int tdfa_vocab_destroy(tdfa_vocab* v)
{
    if (!v) return TDFA_OK;
    if (v->words) (void)hipFree(v->words);
    if (v->off) (void)hipFree(v->off);
    if (v->len) (void)hipFree(v->len);
    if (v->sorted) (void)hipFree(v->sorted);
    if (v->prefix) (void)hipFree(v->prefix);
    for (int lvl = 0; lvl < 2; ++lvl) {
        if (v->group_tokens[lvl]) (void)hipFree(v->group_tokens[lvl]);
        if (v->group_chunks[lvl]) (void)hipFree(v->group_chunks[lvl]);
    }
    if (v->tail_tokens) (void)hipFree(v->tail_tokens);
    delete v;
    return TDFA_OK;
}

int tdfa_vocab_info(const tdfa_vocab* v, int32_t* n_tokens, int64_t* n_bytes, int32_t* max_len)
{
    clear_error();
    if (!v) return fail(TDFA_E_INVALID_ARG, "vocab is NULL");
    if (n_tokens) *n_tokens = v->n_tokens;
    if (n_bytes) *n_bytes = v->n_bytes;
    if (max_len) *max_len = v->max_len;
    return TDFA_OK;
}

int tdfa_dfa_create(const int32_t* trans, const uint8_t* accept, int32_t n_states, int32_t start, void* stream,
                    tdfa_dfa** out)
{
    clear_error();
    if (!out) return fail(TDFA_E_INVALID_ARG, "out is NULL");
    *out = nullptr;
    if (!trans) return fail(TDFA_E_INVALID_ARG, "trans is NULL");
    if (n_states <= 0 || n_states > (1 << 22) - 64)
        return fail(TDFA_E_INVALID_ARG, "n_states %d outside [1, 2^22 - 64]", n_states);   // table offsets stay below 2^32
    if (start < 0 || start >= n_states) return fail(TDFA_E_INVALID_ARG, "start %d outside [0, %d)", start, n_states);
    // Range check, lane order and jump tables (host, one pass over the table per step).
    tdfa::StatePlan plan;
    {
        const int prc = tdfa::make_state_plan(trans, n_states, &plan);
        if (prc != TDFA_OK) return prc;
    }

    tdfa_dfa* d = new (std::nothrow) tdfa_dfa;
    if (!d) return fail(TDFA_E_OOM, "host allocation failed");
    d->n_states = n_states;
    d->start = start;
    d->q_stride = (n_states + 1 + 63) / 64 * 64;          // room for the sink state after the real ones
    d->narrow = d->q_stride <= 32768;                     // every byte offset state * 2 fits 16 bits
    d->n_order = (int32_t)plan.order.size();
    d->has_jump = plan.n_classes > 0;
    d->n_pairs = plan.n_pairs;
    hipStream_t s = static_cast<hipStream_t>(stream);
    std::vector<uint8_t> acc;
    std::vector<unsigned char> blob;
    int rc = TDFA_OK;
    try {
        // the plan as the kernel reads it (layout in tdfa_internal.h); jump tables in offset form
        const size_t esz = d->narrow ? 2 : 4;
        const size_t jump_off = tdfa::plan_jump_offset(d->n_order);
        blob.assign(jump_off + (plan.n_classes ? (size_t)tdfa::kJumpDepth * d->q_stride * esz : 0), 0);
        if (plan.n_classes) memcpy(blob.data(), plan.clean_set.data(), plan.clean_set.size() * 4);
        memcpy(blob.data() + tdfa::kPlanSetBytes, plan.group_class.data(), plan.group_class.size());
        memcpy(blob.data() + tdfa::plan_live_offset(d->n_order), plan.group_live.data(), plan.group_live.size() * 4);
        if (plan.n_classes) {
            const uint32_t sink = (uint32_t)(d->q_stride - 1);
            tdfa::host_tasks((unsigned)tdfa::kJumpDepth, [&](unsigned m) {        // a row of the jump table per task
                unsigned char* row = blob.data() + jump_off + (size_t)m * d->q_stride * esz;
                const int32_t* src = plan.jump.data() + (size_t)m * n_states;
                if (d->narrow) {
                    uint16_t* out16 = reinterpret_cast<uint16_t*>(row);
                    for (int32_t q = 0; q < n_states; ++q) out16[q] = (uint16_t)((src[q] >= 0 ? (uint32_t)src[q] : sink) * 2);
                    for (int32_t q = n_states; q < d->q_stride; ++q) out16[q] = (uint16_t)(sink * 2);
                } else {
                    uint32_t* out32 = reinterpret_cast<uint32_t*>(row);
                    for (int32_t q = 0; q < n_states; ++q) out32[q] = (src[q] >= 0 ? (uint32_t)src[q] : sink) * 4;
                    for (int32_t q = n_states; q < d->q_stride; ++q) out32[q] = sink * 4;
                }
            });
        }
        plan.jump.clear();
        plan.jump.shrink_to_fit();
    } catch (const std::bad_alloc&) {
        rc = fail(TDFA_E_OOM, "host allocation failed");
    }
    if (rc == TDFA_OK) rc = dfa_alloc(d, &d->trans, (size_t)n_states * 256);
    if (rc == TDFA_OK) rc = dfa_alloc(d, &d->accept, (size_t)n_states);
    if (rc == TDFA_OK) rc = dfa_alloc(d, &d->order, (size_t)d->n_order);
    if (rc == TDFA_OK) rc = dfa_alloc(d, &d->plan, blob.size());
    if (rc == TDFA_OK) {
        unsigned char* tt = nullptr;
        rc = dfa_alloc(d, &tt, (size_t)256 * d->q_stride * (d->narrow ? 2 : 4));
        d->trans_t = tt;
    }
    // the copies go on a stream of the library's own: the call waits for them, not for the caller's stream
    (void)s;
    hipStream_t up = nullptr;
    if (rc == TDFA_OK) rc = upload_stream(&up);
    if (rc == TDFA_OK) {
        try {
            acc.assign((size_t)n_states, 0);
        } catch (const std::bad_alloc&) {
            rc = fail(TDFA_E_OOM, "host allocation failed");
        }
    }
    if (rc == TDFA_OK) {
        if (accept)
            for (int32_t q = 0; q < n_states; ++q) acc[q] = accept[q] ? 1 : 0;
        hipError_t e = hipMemcpyAsync(d->trans, trans, (size_t)n_states * 1024, hipMemcpyHostToDevice, up);
        if (e == hipSuccess) e = hipMemcpyAsync(d->accept, acc.data(), (size_t)n_states, hipMemcpyHostToDevice, up);
        if (e == hipSuccess) e = hipMemcpyAsync(d->order, plan.order.data(), (size_t)d->n_order * 4, hipMemcpyHostToDevice, up);
        if (e == hipSuccess) e = hipMemcpyAsync(d->plan, blob.data(), blob.size(), hipMemcpyHostToDevice, up);
        if (e == hipSuccess) e = hipStreamSynchronize(up);
        if (e != hipSuccess) rc = fail(TDFA_E_DEVICE, "upload: %s", hipGetErrorString(e));
    }
    if (rc != TDFA_OK) {
        tdfa_dfa_destroy(d);
        return rc;
    }
    *out = d;
    return TDFA_OK;
}

int tdfa_dfa_union_host(const int32_t* const* trans, const uint8_t* const* accept, const int32_t* n_states, int32_t n, int32_t start,
                        void* stream, tdfa_dfa** out, int64_t* row_offsets_host)
{
    clear_error();
    if (!out) return fail(TDFA_E_INVALID_ARG, "out is NULL");
    *out = nullptr;
    if (!trans || !n_states || n < 1 || !row_offsets_host) return fail(TDFA_E_INVALID_ARG, "trans / n_states / row_offsets_host NULL or n < 1");
    int64_t total = 0;
    for (int32_t c = 0; c < n; ++c) {
        if (!trans[c] || n_states[c] <= 0) return fail(TDFA_E_INVALID_ARG, "automaton %d: trans is NULL or it has no state", c);
        row_offsets_host[c] = total;
        total += n_states[c];
    }
    row_offsets_host[n] = total;
    if (total > (1 << 22) - 64) return fail(TDFA_E_INVALID_ARG, "the union has %lld states, more than 2^22 - 64", (long long)total);
    if (start < 0 || start >= n_states[0]) return fail(TDFA_E_INVALID_ARG, "start %d outside [0, %d)", start, n_states[0]);
    std::vector<int32_t> all;
    std::vector<uint8_t> acc;
    try {
        all.resize((size_t)total * 256);
        acc.assign((size_t)total, 0);
    } catch (const std::bad_alloc&) {
        return fail(TDFA_E_OOM, "host allocation failed");
    }
    // each automaton's rows with its offset added to the live entries (entries out of range stay out
    // of range or become so, and tdfa_dfa_create names them)
    tdfa::host_tasks((unsigned)n, [&](unsigned c) {
        const int32_t base = (int32_t)row_offsets_host[c], ns = n_states[c];
        int32_t* dst = all.data() + (size_t)base * 256;
        const int32_t* src = trans[c];
        for (size_t i = 0; i < (size_t)ns * 256; ++i) {
            const int32_t to = src[i];
            dst[i] = to >= 0 && to < ns ? to + base : (to == TDFA_DEAD ? TDFA_DEAD : INT32_MIN);
        }
        if (accept && accept[c])
            for (int32_t q = 0; q < ns; ++q) acc[(size_t)base + (size_t)q] = accept[c][q] ? 1 : 0;
    });
    return tdfa_dfa_create(all.data(), acc.data(), (int32_t)total, start, stream, out);
}

int tdfa_dfa_union(const tdfa_dfa* const* dfas, int32_t n, void* stream, tdfa_dfa** out, int64_t* row_offsets_host)
{
    clear_error();
    if (!out) return fail(TDFA_E_INVALID_ARG, "out is NULL");
    *out = nullptr;
    if (!dfas || n < 1 || !row_offsets_host) return fail(TDFA_E_INVALID_ARG, "dfas / row_offsets_host NULL or n < 1");
    int64_t total = 0;
    for (int32_t c = 0; c < n; ++c) {
        if (!dfas[c]) return fail(TDFA_E_INVALID_ARG, "dfas[%d] is NULL", c);
        row_offsets_host[c] = total;
        total += dfas[c]->n_states;
    }
    row_offsets_host[n] = total;
    if (total > (1 << 22) - 64) return fail(TDFA_E_INVALID_ARG, "the union has %lld states, more than 2^22 - 64", (long long)total);
    std::vector<int32_t> trans;
    std::vector<uint8_t> accept;
    try {
        trans.resize((size_t)total * 256);
        accept.resize((size_t)total);
    } catch (const std::bad_alloc&) {
        return fail(TDFA_E_OOM, "host allocation failed");
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    for (int32_t c = 0; c < n; ++c) {
        int32_t* dst = trans.data() + (size_t)row_offsets_host[c] * 256;
        TDFA_HIP(hipMemcpyAsync(dst, dfas[c]->trans, (size_t)dfas[c]->n_states * 1024, hipMemcpyDeviceToHost, s));
        TDFA_HIP(hipMemcpyAsync(accept.data() + row_offsets_host[c], dfas[c]->accept, (size_t)dfas[c]->n_states,
                                hipMemcpyDeviceToHost, s));
    }
    TDFA_HIP(hipStreamSynchronize(s));
    for (int32_t c = 0; c < n; ++c) {
        const int32_t base = (int32_t)row_offsets_host[c];
        int32_t* dst = trans.data() + (size_t)base * 256;
        const size_t count = (size_t)dfas[c]->n_states * 256;
        for (size_t i = 0; i < count; ++i)
            if (dst[i] >= 0) dst[i] += base;
    }
    return tdfa_dfa_create(trans.data(), accept.data(), (int32_t)total, dfas[0]->start, stream, out);
}

int tdfa_plan_describe(const int32_t* trans, int32_t n_states, int32_t* order, int32_t cap, int32_t* n_order,
                       int8_t* group_class, uint32_t* clean_sets, int32_t* jump, int32_t* n_classes)
{
    clear_error();
    if (!trans || !order || !n_order || !group_class || !clean_sets || !n_classes)
        return fail(TDFA_E_INVALID_ARG, "NULL argument");
    if (n_states <= 0 || n_states > (1 << 22) - 64)
        return fail(TDFA_E_INVALID_ARG, "n_states %d outside [1, 2^22 - 64]", n_states);
    tdfa::StatePlan plan;
    const int rc = tdfa::make_state_plan(trans, n_states, &plan);
    if (rc != TDFA_OK) return rc;
    *n_order = (int32_t)plan.order.size();
    *n_classes = plan.n_classes;
    if ((size_t)cap < plan.order.size()) return fail(TDFA_E_INVALID_ARG, "order holds %d entries, %zu needed", cap, plan.order.size());
    memcpy(order, plan.order.data(), plan.order.size() * 4);
    memcpy(group_class, plan.group_class.data(), plan.group_class.size());
    memset(clean_sets, 0, (size_t)tdfa::kMaxJumpClasses * 32);
    memcpy(clean_sets, plan.clean_set.data(), plan.clean_set.size() * 4);
    if (jump) {
        for (size_t i = 0; i < (size_t)tdfa::kJumpDepth * (size_t)n_states; ++i) jump[i] = TDFA_DEAD;
        if (plan.n_classes) memcpy(jump, plan.jump.data(), plan.jump.size() * 4);
    }
    return TDFA_OK;
}

int tdfa_dfa_workspace_limit(tdfa_dfa* d, int64_t max_bytes)
{
    clear_error();
    if (!d) return fail(TDFA_E_INVALID_ARG, "dfa is NULL");
    if (max_bytes < 0) return fail(TDFA_E_INVALID_ARG, "max_bytes %lld is negative", (long long)max_bytes);
    d->start_limit = (size_t)max_bytes;
    return TDFA_OK;
}

int tdfa_trim(void)
{
    clear_error();
    std::vector<void*> to_free;
    {
        std::lock_guard<std::mutex> lock(tdfa::g_pool_mutex);
        for (const tdfa::PoolBlock& b : tdfa::g_pool) to_free.push_back(b.ptr);
        tdfa::g_pool.clear();
    }
    for (void* p : to_free) (void)hipFree(p);
    tdfa::cache_trim();
    return TDFA_OK;
}

int tdfa_dfa_info(const tdfa_dfa* d, int32_t* n_states, int32_t* start, int32_t* compile_path, int64_t* workspace_bytes)
{
    clear_error();
    if (!d) return fail(TDFA_E_INVALID_ARG, "dfa is NULL");
    if (n_states) *n_states = d->n_states;
    if (start) *start = d->start;
    const bool pairs = takes_pairs(d);
    const bool staged = !pairs && d->path == TDFA_PATH_STAGED && d->narrow && (size_t)256 * d->q_stride * 2 <= tdfa::kStagedTableBytes;
    if (compile_path) *compile_path = pairs ? TDFA_PATH_PAIRS : staged ? TDFA_PATH_STAGED : TDFA_PATH_WALK;
    if (workspace_bytes)
        *workspace_bytes = pairs && d->sweep.sized ? (int64_t)((d->sweep.list2_cap + 2 * d->sweep.buf_cap) * 4) : -1;
    return TDFA_OK;
}

int tdfa_dfa_compile_path(tdfa_dfa* d, int path)
{
    clear_error();
    if (!d) return fail(TDFA_E_INVALID_ARG, "dfa is NULL");
    if (path != TDFA_PATH_AUTO && path != TDFA_PATH_WALK && path != TDFA_PATH_PAIRS && path != TDFA_PATH_STAGED)
        return fail(TDFA_E_INVALID_ARG, "unknown path %d", path);
    d->path = path;
    return TDFA_OK;
}

int tdfa_dfa_destroy(tdfa_dfa* d)
{
    if (!d) return TDFA_OK;
    free_sweep(&d->sweep);
    // the table, the plan and the walk's workspace go to the cache with the event of the last compile call that
    // used them; after a launch under stream capture no event can say when the GPU is done: then wait for it
    if (d->used_in_capture) (void)hipDeviceSynchronize();
    for (const std::pair<void*, size_t>& b : d->cached) tdfa::cache_free(b.first, b.second, d->used_in_capture ? nullptr : d->used);
    delete d;
    return TDFA_OK;
}

int tdfa_compile_token_dfa(const tdfa_vocab* vocab, const tdfa_dfa* dfa, int32_t* delta_dev, uint32_t* allow_dev,
                           void* stream, tdfa_table** out)
{
    return tdfa_compile_token_dfa_at(vocab, dfa, 0, delta_dev, allow_dev, stream, out);
}

int tdfa_compile_token_dfa_at(const tdfa_vocab* vocab, const tdfa_dfa* dfa, int64_t row_base, int32_t* delta_dev,
                              uint32_t* allow_dev, void* stream, tdfa_table** out)
{
    clear_error();
    if (!out) return fail(TDFA_E_INVALID_ARG, "out is NULL");
    *out = nullptr;
    if (!vocab || !dfa) return fail(TDFA_E_INVALID_ARG, "vocab or dfa is NULL");
    if (row_base < 0 || row_base + dfa->n_states > 0x7FFFFFFFll)
        return fail(TDFA_E_INVALID_ARG, "row_base %lld puts states outside int32", (long long)row_base);
    tdfa_table* t = nullptr;
    int rc = make_table(dfa->n_states, vocab->n_tokens, delta_dev, allow_dev, &t);
    if (rc != TDFA_OK) return rc;
    CompileEntry e;
    rc = before_use(dfa, static_cast<hipStream_t>(stream));
    if (rc == TDFA_OK) rc = entry_of(dfa, vocab, 0, (int32_t)row_base, static_cast<hipStream_t>(stream), &e);
    CompileArgs a = args_of(vocab, t, &e, 1);
    if (rc == TDFA_OK) rc = launch_compile(a, static_cast<hipStream_t>(stream));
    {
        const int urc = after_use(&dfa, 1, static_cast<hipStream_t>(stream));       // (also behind launches of a call that failed half-way)
        if (rc == TDFA_OK) rc = urc;
    }
    if (rc == TDFA_OK) rc = count_rows(t, static_cast<hipStream_t>(stream));
    if (rc != TDFA_OK) {
        tdfa_table_destroy(t);
        return rc;
    }
    *out = t;
    return TDFA_OK;
}

int tdfa_compile_stacked(const tdfa_vocab* vocab, const tdfa_dfa* const* dfas, int32_t n, int32_t* delta_dev,
                         uint32_t* allow_dev, void* stream, tdfa_table** out, int64_t* row_offsets_host)
{
    clear_error();
    if (!out) return fail(TDFA_E_INVALID_ARG, "out is NULL");
    *out = nullptr;
    if (!vocab || !dfas || n < 1 || !row_offsets_host) return fail(TDFA_E_INVALID_ARG, "vocab / dfas / row_offsets_host NULL or n < 1");
    std::vector<CompileEntry> entries;
    try {
        entries.reserve((size_t)n);
    } catch (const std::bad_alloc&) {
        return fail(TDFA_E_OOM, "host allocation failed");
    }
    int64_t rows = 0;
    for (int32_t c = 0; c < n; ++c) {
        if (!dfas[c]) return fail(TDFA_E_INVALID_ARG, "dfas[%d] is NULL", c);
        row_offsets_host[c] = rows;
        if (rows + dfas[c]->n_states > 0x7FFFFFFFll) return fail(TDFA_E_UNSUPPORTED, "more than 2^31 rows");
        CompileEntry e;
        int erc = before_use(dfas[c], static_cast<hipStream_t>(stream));
        if (erc == TDFA_OK) erc = entry_of(dfas[c], vocab, (int32_t)rows, (int32_t)rows, static_cast<hipStream_t>(stream), &e);
        if (erc != TDFA_OK) {
            (void)after_use(dfas, c + 1, static_cast<hipStream_t>(stream));        // (entry_of may have launched the sweep's sizing kernels)
            return erc;
        }
        entries.push_back(e);
        rows += dfas[c]->n_states;
    }
    row_offsets_host[n] = rows;
    tdfa_table* t = nullptr;
    int rc = make_table(rows, vocab->n_tokens, delta_dev, allow_dev, &t);
    if (rc != TDFA_OK) {
        (void)after_use(dfas, n, static_cast<hipStream_t>(stream));
        return rc;
    }
    CompileArgs a = args_of(vocab, t, entries.data(), n);
    rc = launch_compile(a, static_cast<hipStream_t>(stream));
    {
        const int urc = after_use(dfas, n, static_cast<hipStream_t>(stream));
        if (rc == TDFA_OK) rc = urc;
    }
    if (rc == TDFA_OK) rc = count_rows(t, static_cast<hipStream_t>(stream));
    if (rc != TDFA_OK) {
        tdfa_table_destroy(t);
        return rc;
    }
    *out = t;
    return TDFA_OK;
}

int tdfa_table_concat(const tdfa_table* const* tables, int32_t n, int32_t* delta_dev, uint32_t* allow_dev,
                      void* stream, tdfa_table** out, int64_t* row_offsets_host)
{
    clear_error();
    if (!out) return fail(TDFA_E_INVALID_ARG, "out is NULL");
    *out = nullptr;
    if (!tables || n < 1 || !row_offsets_host) return fail(TDFA_E_INVALID_ARG, "tables / row_offsets_host NULL or n < 1");
    int64_t rows = 0;
    for (int32_t c = 0; c < n; ++c) {
        if (!tables[c]) return fail(TDFA_E_INVALID_ARG, "tables[%d] is NULL", c);
        if (!tables[c]->delta) return fail(TDFA_E_INVALID_ARG, "tables[%d] is packed; stack dense tables, then pack", c);
        if (tables[c]->n_tokens != tables[0]->n_tokens)
            return fail(TDFA_E_INVALID_ARG, "tables[%d] has %d tokens, tables[0] has %d", c, tables[c]->n_tokens,
                        tables[0]->n_tokens);
        row_offsets_host[c] = rows;
        rows += tables[c]->n_rows;
    }
    row_offsets_host[n] = rows;
    if (rows > 0x7FFFFFFFll) return fail(TDFA_E_UNSUPPORTED, "more than 2^31 rows");
    tdfa_table* t = nullptr;
    int rc = make_table(rows, tables[0]->n_tokens, delta_dev, allow_dev, &t);
    if (rc != TDFA_OK) return rc;
    for (int32_t c = 0; c < n && rc == TDFA_OK; ++c)
        rc = launch_concat_part(tables[c]->delta, tables[c]->allow, tables[c]->n_rows, t->n_tokens, t->row_words,
                                row_offsets_host[c], t->delta, t->allow, static_cast<hipStream_t>(stream));
    if (rc == TDFA_OK) rc = count_rows(t, static_cast<hipStream_t>(stream));
    if (rc != TDFA_OK) {
        tdfa_table_destroy(t);
        return rc;
    }
    *out = t;
    return TDFA_OK;
}

int tdfa_table_wrap(int32_t* delta_dev, uint32_t* allow_dev, int64_t n_rows, int32_t n_tokens, tdfa_table** out)
{
    clear_error();
    if (!out) return fail(TDFA_E_INVALID_ARG, "out is NULL");
    *out = nullptr;
    if (!delta_dev || !allow_dev) return fail(TDFA_E_INVALID_ARG, "delta_dev or allow_dev is NULL");
    if (n_rows < 0 || n_rows > 0x7FFFFFFFll || n_tokens < 0) return fail(TDFA_E_INVALID_ARG, "bad table shape");
    return make_table(n_rows, n_tokens, delta_dev, allow_dev, out);
}

int tdfa_table_info(const tdfa_table* t, int64_t* n_rows, int32_t* n_tokens, int32_t** delta_dev,
                    uint32_t** allow_dev, int64_t* allow_row_words_out)
{
    clear_error();
    if (!t) return fail(TDFA_E_INVALID_ARG, "table is NULL");
    if (n_rows) *n_rows = t->n_rows;
    if (n_tokens) *n_tokens = t->n_tokens;
    if (delta_dev) *delta_dev = t->delta;
    if (allow_dev) *allow_dev = t->allow;
    if (allow_row_words_out) *allow_row_words_out = t->row_words;
    return TDFA_OK;
}

int tdfa_table_destroy(tdfa_table* t)
{
    if (!t) return TDFA_OK;
    tdfa::pool_release(t->row_allowed);
    if (t->own_delta && t->delta) (void)hipFree(t->delta);
    if (t->own_allow && t->allow) (void)hipFree(t->allow);
    if (t->targets) (void)hipFree(t->targets);
    if (t->row_begin) (void)hipFree(t->row_begin);
    if (t->dir) (void)hipFree(t->dir);
    delete t;
    return TDFA_OK;
}

namespace {

void fill_table_args(const tdfa_table* table, tdfa::MaskArgs* a)
{
    a->delta = table->delta;
    a->targets = table->targets;
    a->row_begin = table->row_begin;
    a->dir = table->dir;
    a->allow = table->allow;
    a->row_allowed = table->row_allowed;
    a->n_rows = table->n_rows;
    a->n_tokens = table->n_tokens;
    a->row_words = table->row_words;
}

// Argument checks and kernel arguments shared by the greedy and the sampling step.
int prepare_step(const tdfa_table* table, const void* logits_dev, int dtype, int32_t batch, int64_t row_stride,
                 const int32_t* states_dev, int32_t* tokens_dev, int32_t* new_states_dev, void* masked_out_dev,
                 hipStream_t s, tdfa::MaskArgs* a, uint32_t** words_scratch = nullptr, bool use_static = false)
{
    if (!table) return fail(TDFA_E_INVALID_ARG, "table is NULL");
    if (dtype != TDFA_F32 && dtype != TDFA_BF16) return fail(TDFA_E_INVALID_ARG, "unknown dtype %d", dtype);
    if (batch < 0) return fail(TDFA_E_INVALID_ARG, "batch %d is negative", batch);
    if (batch == 0) return TDFA_OK;
    if (!logits_dev || !states_dev || !tokens_dev || !new_states_dev)
        return fail(TDFA_E_INVALID_ARG, "logits, states, tokens or new_states is NULL");
    if (row_stride < table->n_tokens) return fail(TDFA_E_INVALID_ARG, "row_stride %lld < n_tokens %d", (long long)row_stride, table->n_tokens);
    const int64_t esz = dtype == TDFA_F32 ? 4 : 2;
    if ((reinterpret_cast<uintptr_t>(logits_dev) & 15) || ((row_stride * esz) & 15) ||
        (reinterpret_cast<uintptr_t>(masked_out_dev) & 15))
        return fail(TDFA_E_INVALID_ARG, "logits / masked_out rows must be 16-byte aligned");
    DeviceScratch sc;
    if (use_static) {
        // no allocation on this path: the fixed array in the device image, for batches that fit it
        if (batch > kStaticMaxBatch)
            return fail(TDFA_E_UNSUPPORTED, "batch %d exceeds the %d sequences the static scratch holds", batch, kStaticMaxBatch);
        void* ptr = nullptr;
        const int src = static_scratch(&ptr);
        if (src != TDFA_OK) return src;
        sc.best = static_cast<unsigned long long*>(ptr);
        sc.count = reinterpret_cast<unsigned int*>(static_cast<unsigned char*>(ptr) + (size_t)kStaticMaxBatch * sizeof(unsigned long long));
        sc.cap = kStaticMaxBatch;
    } else {
        const int rc = ensure_scratch(batch, s, &sc);
        if (rc != TDFA_OK) return rc;
    }
    fill_table_args(table, a);
    a->logits = logits_dev;
    a->dtype = dtype;
    a->batch = batch;
    a->row_stride = row_stride;
    a->states = states_dev;
    a->tokens = tokens_dev;
    a->new_states = new_states_dev;
    a->masked_out = masked_out_dev;
    a->scratch_best = sc.best;
    a->scratch_count = sc.count;
    if (words_scratch) *words_scratch = use_static ? nullptr : sc.count + sc.cap;
    return TDFA_OK;
}

}  // namespace

int tdfa_mask_step(const tdfa_table* table, const void* logits_dev, int dtype, int32_t batch, int64_t row_stride,
                   const int32_t* states_dev, int32_t* tokens_dev, int32_t* new_states_dev, void* masked_out_dev,
                   void* stream)
{
    clear_error();
    hipStream_t s = static_cast<hipStream_t>(stream);
    MaskArgs a = {};
    a.batch = 0;
    int rc = prepare_step(table, logits_dev, dtype, batch, row_stride, states_dev, tokens_dev, new_states_dev,
                          masked_out_dev, s, &a);
    if (rc != TDFA_OK || batch == 0) return rc;
    return launch_mask_step(a, s);
}

int tdfa_mask_step_noalloc(const tdfa_table* table, const void* logits_dev, int dtype, int32_t batch, int64_t row_stride,
                           const int32_t* states_dev, int32_t* tokens_dev, int32_t* new_states_dev, void* masked_out_dev,
                           void* stream)
{
    clear_error();
    hipStream_t s = static_cast<hipStream_t>(stream);
    MaskArgs a = {};
    a.batch = 0;
    int rc = prepare_step(table, logits_dev, dtype, batch, row_stride, states_dev, tokens_dev, new_states_dev,
                          masked_out_dev, s, &a, nullptr, true);
    if (rc != TDFA_OK || batch == 0) return rc;
    // The array is shared by every call on this GPU and keeps what the last one left: the words this
    // call's workgroups meet through are cleared first, by a kernel (a recorded graph may hold this).
    if (mask_step_uses_scratch(a)) {
        rc = launch_clear_scratch(a.scratch_best, a.scratch_count, batch, s);
        if (rc != TDFA_OK) return rc;
    }
    return launch_mask_step(a, s);
}

namespace {

int sample_step_impl(const tdfa_table* table, const void* logits_dev, int dtype, int32_t batch, int64_t row_stride,
                     const int32_t* states_dev, float temperature, int32_t top_k, uint64_t seed, uint64_t offset,
                     const uint64_t* offset_dev, int32_t* tokens_dev, int32_t* new_states_dev, void* masked_out_dev,
                     void* stream)
{
    if (!(temperature > 0.0f)) return fail(TDFA_E_INVALID_ARG, "temperature %g is not positive", (double)temperature);
    if (top_k < 0) return fail(TDFA_E_INVALID_ARG, "top_k %d is negative", top_k);
    const volatile float one = 1.0f;                     // divided at run time, rounded once to binary32
    const float inv_t = one / temperature;
    if (!(inv_t > 0.0f) || inv_t > 3.402823466e38f)
        return fail(TDFA_E_INVALID_ARG, "1 / temperature is not finite for temperature %g", (double)temperature);
    hipStream_t s = static_cast<hipStream_t>(stream);
    MaskArgs a = {};
    a.batch = 0;
    uint32_t* cut = nullptr;
    int rc = prepare_step(table, logits_dev, dtype, batch, row_stride, states_dev, tokens_dev, new_states_dev,
                          masked_out_dev, s, &a, &cut);
    if (rc != TDFA_OK || batch == 0) return rc;
    return launch_sample_step(a, inv_t, top_k, cut, seed, offset, offset_dev, s);
}

}  // namespace

int tdfa_sample_step(const tdfa_table* table, const void* logits_dev, int dtype, int32_t batch, int64_t row_stride,
                     const int32_t* states_dev, float temperature, int32_t top_k, uint64_t seed, uint64_t offset,
                     int32_t* tokens_dev, int32_t* new_states_dev, void* masked_out_dev, void* stream)
{
    clear_error();
    return sample_step_impl(table, logits_dev, dtype, batch, row_stride, states_dev, temperature, top_k, seed, offset,
                            nullptr, tokens_dev, new_states_dev, masked_out_dev, stream);
}

int tdfa_sample_step_at(const tdfa_table* table, const void* logits_dev, int dtype, int32_t batch, int64_t row_stride,
                        const int32_t* states_dev, float temperature, int32_t top_k, uint64_t seed,
                        const uint64_t* offset_dev, int32_t* tokens_dev, int32_t* new_states_dev, void* masked_out_dev,
                        void* stream)
{
    clear_error();
    if (!offset_dev) return fail(TDFA_E_INVALID_ARG, "offset_dev is NULL");
    if (reinterpret_cast<uintptr_t>(offset_dev) & 7) return fail(TDFA_E_INVALID_ARG, "offset_dev must be 8-byte aligned");
    return sample_step_impl(table, logits_dev, dtype, batch, row_stride, states_dev, temperature, top_k, seed, 0,
                            offset_dev, tokens_dev, new_states_dev, masked_out_dev, stream);
}

int tdfa_sample_noise(int32_t batch, int32_t n_tokens, uint64_t seed, uint64_t offset, float* noise_dev, void* stream)
{
    clear_error();
    if (batch < 0 || n_tokens < 0) return fail(TDFA_E_INVALID_ARG, "batch %d or n_tokens %d is negative", batch, n_tokens);
    if (batch == 0 || n_tokens == 0) return TDFA_OK;
    if (!noise_dev) return fail(TDFA_E_INVALID_ARG, "noise is NULL");
    return launch_sample_noise(batch, n_tokens, seed, offset, noise_dev, static_cast<hipStream_t>(stream));
}

int tdfa_table_apply_terminals(tdfa_table* table, int32_t n_edges, const int32_t* edge_state_host,
                               const int32_t* edge_label_host, const int32_t* edge_target_host, int32_t n_labels,
                               const uint32_t* masks_dev, void* stream)
{
    clear_error();
    if (!table) return fail(TDFA_E_INVALID_ARG, "table is NULL");
    if (!table->delta) return fail(TDFA_E_INVALID_ARG, "the table is packed; apply terminal edges to the dense table, then pack");
    if (n_edges < 0 || n_labels < 0) return fail(TDFA_E_INVALID_ARG, "n_edges %d or n_labels %d is negative", n_edges, n_labels);
    if (n_edges == 0) return TDFA_OK;
    if (!edge_state_host || !edge_label_host || !edge_target_host || !masks_dev)
        return fail(TDFA_E_INVALID_ARG, "edge arrays or masks NULL");
    for (int32_t e = 0; e < n_edges; ++e) {
        if (edge_state_host[e] < 0 || edge_state_host[e] >= table->n_rows || edge_target_host[e] < 0 ||
            edge_target_host[e] >= table->n_rows)
            return fail(TDFA_E_INVALID_ARG, "edge %d: state %d or target %d is not a row of the table", e, edge_state_host[e],
                        edge_target_host[e]);
        if (edge_label_host[e] < 0 || edge_label_host[e] >= n_labels)
            return fail(TDFA_E_INVALID_ARG, "edge %d: label %d outside [0, %d)", e, edge_label_host[e], n_labels);
    }
    // edges by state, the given order kept inside a state: [state_of | edge_begin | label | target]
    std::vector<int32_t> idx, pack;
    int32_t n_u = 0;
    try {
        idx.resize((size_t)n_edges);
        for (int32_t e = 0; e < n_edges; ++e) idx[(size_t)e] = e;
        std::stable_sort(idx.begin(), idx.end(), [&](int32_t x, int32_t y) { return edge_state_host[x] < edge_state_host[y]; });
        for (int32_t i = 0; i < n_edges; ++i)
            if (i == 0 || edge_state_host[idx[(size_t)i]] != edge_state_host[idx[(size_t)i - 1]]) ++n_u;
        pack.resize((size_t)n_u * 2 + 1 + (size_t)n_edges * 2);
        int32_t* state_of = pack.data();
        int32_t* begin = state_of + n_u;
        int32_t* label = begin + n_u + 1;
        int32_t* target = label + n_edges;
        int32_t u = -1;
        for (int32_t i = 0; i < n_edges; ++i) {
            const int32_t e = idx[(size_t)i];
            if (i == 0 || edge_state_host[e] != edge_state_host[idx[(size_t)i - 1]]) {
                ++u;
                state_of[u] = edge_state_host[e];
                begin[u] = i;
            }
            label[i] = edge_label_host[e];
            target[i] = edge_target_host[e];
        }
        begin[n_u] = n_edges;
    } catch (const std::bad_alloc&) {
        return fail(TDFA_E_OOM, "host allocation failed");
    }
    int32_t* dev = nullptr;
    int rc = device_alloc(&dev, pack.size());
    if (rc != TDFA_OK) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipError_t he = hipMemcpyAsync(dev, pack.data(), pack.size() * 4, hipMemcpyHostToDevice, s);
    if (he == hipSuccess) {
        rc = launch_apply_terminals(table->delta, table->allow, table->n_tokens, table->row_words, n_u, dev, dev + n_u,
                                    dev + 2 * (size_t)n_u + 1, dev + 2 * (size_t)n_u + 1 + n_edges, masks_dev, s);
        if (rc == TDFA_OK && table->row_allowed) rc = count_rows(table, s);        // the edges have added allowed tokens
        if (rc == TDFA_OK) he = hipStreamSynchronize(s);
    }
    (void)hipFree(dev);
    if (he != hipSuccess) return fail(TDFA_E_DEVICE, "apply_terminals: %s", hipGetErrorString(he));
    return rc;
}

int tdfa_table_minimize(const tdfa_table* table, const uint8_t* accept_host, const int32_t* start_states_host,
                        int32_t n_starts, void* stream, tdfa_table** out, int32_t* state_map_host, uint8_t* accept_out_host)
{
    clear_error();
    if (!out) return fail(TDFA_E_INVALID_ARG, "out is NULL");
    *out = nullptr;
    if (!table || !accept_host || !start_states_host || !state_map_host)
        return fail(TDFA_E_INVALID_ARG, "table, accept, start states or state map NULL");
    if (!table->delta) return fail(TDFA_E_INVALID_ARG, "the table is packed; minimise the dense table, then pack");
    if (n_starts < 0) return fail(TDFA_E_INVALID_ARG, "n_starts %d is negative", n_starts);
    if (table->n_rows <= 0 || table->n_rows > 0x7FFFFFFFll) return fail(TDFA_E_INVALID_ARG, "the table has no rows or too many");
    for (int32_t i = 0; i < n_starts; ++i)
        if (start_states_host[i] < 0 || start_states_host[i] >= table->n_rows)
            return fail(TDFA_E_INVALID_ARG, "start state %d is not a row of the table", start_states_host[i]);
    hipStream_t s = static_cast<hipStream_t>(stream);
    std::vector<int32_t> first_rows, map;
    int rc;
    try {
        rc = minimize_table(table->delta, table->n_rows, table->n_tokens, accept_host, start_states_host, n_starts, s,
                            &first_rows, &map);
    } catch (const std::bad_alloc&) {
        return fail(TDFA_E_OOM, "host allocation failed");
    }
    if (rc != TDFA_OK) return rc;
    tdfa_table* t = nullptr;
    rc = make_table((int64_t)first_rows.size(), table->n_tokens, nullptr, nullptr, &t);
    if (rc != TDFA_OK) return rc;
    rc = launch_compact_rows(table->delta, table->n_tokens, table->row_words, first_rows, map, t->delta, t->allow, s);
    if (rc == TDFA_OK) rc = count_rows(t, s);
    if (rc != TDFA_OK) {
        tdfa_table_destroy(t);
        return rc;
    }
    memcpy(state_map_host, map.data(), map.size() * 4);
    if (accept_out_host)
        for (size_t c = 0; c < first_rows.size(); ++c) accept_out_host[c] = accept_host[first_rows[c]] ? 1 : 0;
    *out = t;
    return TDFA_OK;
}

int tdfa_advance_tokens(const tdfa_table* table, int32_t batch, int32_t k, const int32_t* states_dev,
                        const int32_t* tokens_dev, int32_t* history_dev, int32_t* n_valid_dev, void* stream)
{
    clear_error();
    if (!table) return fail(TDFA_E_INVALID_ARG, "table is NULL");
    if (batch < 0 || k < 0) return fail(TDFA_E_INVALID_ARG, "batch %d or k %d is negative", batch, k);
    if (batch == 0) return TDFA_OK;
    if (!states_dev || !history_dev || (k > 0 && !tokens_dev))
        return fail(TDFA_E_INVALID_ARG, "states, tokens or history is NULL");
    MaskArgs a = {};
    fill_table_args(table, &a);
    return launch_advance_tokens(a, batch, k, states_dev, tokens_dev, history_dev, n_valid_dev,
                                 static_cast<hipStream_t>(stream));
}

int tdfa_table_pack(const tdfa_table* table, void* stream, tdfa_table** out)
{
    clear_error();
    if (!out) return fail(TDFA_E_INVALID_ARG, "out is NULL");
    *out = nullptr;
    if (!table) return fail(TDFA_E_INVALID_ARG, "table is NULL");
    if (!table->delta) return fail(TDFA_E_INVALID_ARG, "the table is packed already");
    if (reinterpret_cast<uintptr_t>(table->allow) & 15) return fail(TDFA_E_INVALID_ARG, "allowed-bit rows must be 16-byte aligned");
    hipStream_t s = static_cast<hipStream_t>(stream);
    tdfa_table* t = new (std::nothrow) tdfa_table;
    if (!t) return fail(TDFA_E_OOM, "host allocation failed");
    t->n_rows = table->n_rows;
    t->n_tokens = table->n_tokens;
    t->row_words = table->row_words;
    int rc = device_alloc(&t->allow, (size_t)t->n_rows * (size_t)t->row_words);
    t->own_allow = rc == TDFA_OK;
    if (rc == TDFA_OK && t->n_rows > 0 && t->row_words > 0) {
        hipError_t e = hipMemcpyAsync(t->allow, table->allow, (size_t)t->n_rows * (size_t)t->row_words * sizeof(uint32_t),
                                      hipMemcpyDeviceToDevice, s);
        if (e != hipSuccess) rc = fail(TDFA_E_DEVICE, "copy of the allowed bits: %s", hipGetErrorString(e));
    }
    if (rc == TDFA_OK)
        rc = pack_table(table->delta, table->allow, t->n_rows, t->n_tokens, t->row_words, s, &t->dir, &t->row_begin,
                        &t->targets, &t->n_edges);
    if (rc != TDFA_OK) {
        (void)hipStreamSynchronize(s);
        tdfa_table_destroy(t);
        return rc;
    }
    *out = t;
    return TDFA_OK;
}

int tdfa_table_pack_info(const tdfa_table* t, int64_t* n_edges, int32_t** targets_dev, int64_t** row_begin_dev,
                         uint32_t** dir_dev, int64_t* dir_row_entries)
{
    clear_error();
    if (!t) return fail(TDFA_E_INVALID_ARG, "table is NULL");
    if (t->delta) return fail(TDFA_E_INVALID_ARG, "the table is not packed");
    if (n_edges) *n_edges = t->n_edges;
    if (targets_dev) *targets_dev = t->targets;
    if (row_begin_dev) *row_begin_dev = t->row_begin;
    if (dir_dev) *dir_dev = t->dir;
    if (dir_row_entries) *dir_row_entries = t->row_words / 4;
    return TDFA_OK;
}

}  // extern "C"
