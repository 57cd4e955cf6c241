// Fiber runtime of the host emulation of the HIP kernels (see include/hip/hip_runtime.h): test
// infrastructure, compiled with the library's sources into a host-only shared object.
#include <hip/hip_runtime.h>
#include <sys/mman.h>
#include <ucontext.h>
#include <execinfo.h>
#include <signal.h>
#include <unistd.h>
#include <atomic>
#include <mutex>
#include <thread>
#include <vector>

namespace emu {

struct Wave {
    int arrived = 0;
    unsigned gen = 0;
    const void* ptr[64];
    v4i_t a[64], b[64], c[64];
    int iv[64];
};
struct Fiber {
    ucontext_t ctx;
    dim3 tid;
    int linear = 0;
    bool done = false;
    const char* waiting = "";
    void* stack = nullptr;
};
struct Group {
    std::vector<Fiber> f;
    std::vector<Wave> w;
    ucontext_t sched;
    int current = 0;
    int n = 0;
    int bar_arrived = 0;
    unsigned bar_gen = 0;
    long progress_events = 0;
    dim3 block, grid, bdim;
    const std::function<void()>* fn = nullptr;
};
static thread_local Group* G = nullptr;
static constexpr size_t STACK = 256 * 1024;

Fiber* cur() { return &G->f[G->current]; }
dim3& thread_idx() { return cur()->tid; }
dim3& block_idx() { return G->block; }
dim3& grid_dim() { return G->grid; }
dim3& block_dim() { return G->bdim; }

static void yield_fiber()
{
    Fiber* me = cur();
    swapcontext(&me->ctx, &G->sched);
}
static void progress() { ++G->progress_events; }

void syncthreads()
{
    Fiber* me = cur();
    const unsigned gen = G->bar_gen;
    if (++G->bar_arrived == G->n) {
        G->bar_arrived = 0;
        ++G->bar_gen;
        progress();
        return;
    }
    progress();   // an arrival is a change of state
    me->waiting = "__syncthreads";
    while (G->bar_gen == gen) yield_fiber();
    me->waiting = "";
}
static void wave_sync(Wave& w, const char* what)
{
    Fiber* me = cur();
    const unsigned gen = w.gen;
    if (++w.arrived == 64) {
        w.arrived = 0;
        ++w.gen;
        progress();
        return;
    }
    progress();
    me->waiting = what;
    while (w.gen == gen) yield_fiber();
    me->waiting = "";
}
static Wave& my_wave() { return G->w[cur()->linear >> 6]; }

v2i_t tr8(const void* p)
{
    Wave& w = my_wave();
    const int lane = cur()->linear & 63;
    w.ptr[lane] = p;
    wave_sync(w, "ds_read_tr8 (deposit)");
    const int base = lane & ~15, pp = lane & 15;
    uint8_t out[8];
    for (int t = 0; t < 8; ++t) {
        const uint8_t* src = (const uint8_t*)w.ptr[base + 2 * t + pp / 8];
        out[t] = src[pp % 8];
    }
    wave_sync(w, "ds_read_tr8 (collect)");
    v2i_t r;
    memcpy(&r, out, 8);
    return r;
}
v4i_t mfma_i8_16x16x64(v4i_t a, v4i_t b, v4i_t c)
{
    Wave& w = my_wave();
    const int lane = cur()->linear & 63;
    w.a[lane] = a;
    w.b[lane] = b;
    wave_sync(w, "mfma (deposit)");
    const int g = lane >> 4, col = lane & 15;
    v4i_t d = c;
    for (int r = 0; r < 4; ++r) {
        const int tok = 4 * g + r;
        int32_t s = 0;
        for (int kg = 0; kg < 4; ++kg) {
            int8_t av[16], bv[16];
            memcpy(av, &w.a[kg * 16 + tok], 16);
            memcpy(bv, &w.b[kg * 16 + col], 16);
            for (int t = 0; t < 16; ++t) s += (int32_t)av[t] * (int32_t)bv[t];
        }
        d[r] = (int32_t)((uint32_t)d[r] + (uint32_t)s);
    }
    wave_sync(w, "mfma (collect)");
    return d;
}
void wave_barrier() { wave_sync(my_wave(), "wave_barrier"); }
// swap16: ret0 = [a.row0, b.row0, a.row2, b.row2], ret1 = [a.row1, b.row1, a.row3, b.row3] (rows of 16 lanes);
// swap32: ret0 = [a.lo32, b.lo32], ret1 = [a.hi32, b.hi32]  (as observed on the device)
v2u_t permlane_swap(unsigned a, unsigned b, int rows)
{
    Wave& w = my_wave();
    const int lane = cur()->linear & 63;
    w.iv[lane] = (int)a;
    w.c[lane][0] = (int)b;
    wave_sync(w, "permlane_swap (deposit)");
    v2u_t r;
    if (rows == 16) {
        const int row = lane >> 4, l = lane & 15;
        const int src = (row & 2) * 16 + l;            // row 0 or 2 of the source
        r[0] = (row & 1) ? (unsigned)w.c[src][0] : (unsigned)w.iv[src];
        r[1] = (row & 1) ? (unsigned)w.c[src + 16][0] : (unsigned)w.iv[src + 16];
    } else {
        const int half = lane >> 5, l = lane & 31;
        r[0] = half ? (unsigned)w.c[l][0] : (unsigned)w.iv[l];
        r[1] = half ? (unsigned)w.c[32 + l][0] : (unsigned)w.iv[32 + l];
    }
    wave_sync(w, "permlane_swap (collect)");
    return r;
}
int readfirstlane(int v)
{
    Wave& w = my_wave();
    const int lane = cur()->linear & 63;
    w.iv[lane] = v;
    wave_sync(w, "readfirstlane (deposit)");
    const int r = w.iv[0];
    wave_sync(w, "readfirstlane (collect)");
    return r;
}
int readlane(int v, int src)
{
    Wave& w = my_wave();
    const int lane = cur()->linear & 63;
    w.iv[lane] = v;
    wave_sync(w, "readlane (deposit)");
    const int r = w.iv[src & 63];
    wave_sync(w, "readlane (collect)");
    return r;
}

static void fiber_main()
{
    (*G->fn)();
    cur()->done = true;
    progress();
    swapcontext(&cur()->ctx, &G->sched);
}

static void run_block(Group& g, const std::function<void()>& fn)
{
    G = &g;
    g.fn = &fn;
    g.bar_arrived = 0;
    g.progress_events = 0;
    for (auto& w : g.w) w.arrived = 0;
    for (int i = 0; i < g.n; ++i) {
        Fiber& f = g.f[i];
        f.done = false;
        f.waiting = "";
        getcontext(&f.ctx);
        f.ctx.uc_stack.ss_sp = f.stack;
        f.ctx.uc_stack.ss_size = STACK;
        f.ctx.uc_link = nullptr;
        makecontext(&f.ctx, fiber_main, 0);
    }
    int remaining = g.n, idle_sweeps = 0;
    while (remaining > 0) {
        const long before = g.progress_events;
        remaining = 0;
        for (int i = 0; i < g.n; ++i) {
            if (g.f[i].done) continue;
            ++remaining;
            g.current = i;
            swapcontext(&g.sched, &g.f[i].ctx);
        }
        // a sweep over every live fiber in which no barrier opened, no wave exchange completed and no
        // fiber ended: every live fiber waits for something that cannot happen any more
        idle_sweeps = (g.progress_events == before && remaining > 0) ? idle_sweeps + 1 : 0;
        if (idle_sweeps >= 3) {
            fprintf(stderr, "emu: DEADLOCK in block (%u,%u): %d threads wait; per wave (lane 0):\n", g.block.x, g.block.y, remaining);
            for (int i = 0; i < g.n; i += 64)
                fprintf(stderr, "  wave %d: %s%s\n", i / 64, g.f[i].done ? "finished" : "waiting at ", g.f[i].done ? "" : g.f[i].waiting);
            _exit(86);
        }
    }
}

void launch(dim3 grid, dim3 block, const std::function<void()>& fn)
{
    const int nthreads = (int)(block.x * block.y * block.z);
    if (nthreads % 64 != 0) { fprintf(stderr, "emu: block size %d is not a multiple of 64\n", nthreads); abort(); }
    const long nblocks = (long)grid.x * grid.y * grid.z;
    int workers = 8;
    if (const char* e = getenv("EMU_THREADS")) workers = atoi(e);
    if (workers > nblocks) workers = (int)nblocks;
    std::atomic<long> next{0};
    // EMU_BLOCKS=a,b: run only blocks [a, b) in linear order (x fastest)
    long b0 = 0, b1 = nblocks;
    if (const char* e = getenv("EMU_BLOCKS")) sscanf(e, "%ld,%ld", &b0, &b1);
    next = b0;
    if (b1 > nblocks) b1 = nblocks;
    auto worker = [&]() {
        Group g;
        g.n = nthreads;
        g.f.resize(nthreads);
        g.w.resize(nthreads / 64);
        g.grid = grid;
        g.bdim = block;
        for (int i = 0; i < nthreads; ++i) {
            g.f[i].linear = i;
            g.f[i].tid = dim3(i % block.x, (i / block.x) % block.y, i / (block.x * block.y));
            g.f[i].stack = mmap(nullptr, STACK, PROT_READ | PROT_WRITE, MAP_PRIVATE | MAP_ANONYMOUS | MAP_NORESERVE, -1, 0);
        }
        for (;;) {
            const long b = next.fetch_add(1);
            if (b >= b1) break;
            g.block = dim3((unsigned)(b % grid.x), (unsigned)((b / grid.x) % grid.y), (unsigned)(b / ((long)grid.x * grid.y)));
            run_block(g, fn);
        }
        for (int i = 0; i < nthreads; ++i) munmap(g.f[i].stack, STACK);
    };
    std::vector<std::thread> pool;
    for (int i = 0; i < workers; ++i) pool.emplace_back(worker);
    for (auto& t : pool) t.join();
}

// "device" memory: the allocation ends at a protected page and is preceded by one, so that an
// access past either end is a segmentation fault at the faulting instruction (sizes are rounded
// up to 16 bytes, the granularity of the widest access).
static std::mutex alloc_mu;
struct Alloc { void* base; size_t total; };
static std::vector<std::pair<void*, Alloc>> allocs;
void* dev_alloc(size_t bytes)
{
    const size_t page = (size_t)sysconf(_SC_PAGESIZE);
    const size_t sz = (bytes + 15) & ~(size_t)15;
    const size_t body = (sz + page - 1) / page * page;
    const size_t total = body + 2 * page;
    uint8_t* base = (uint8_t*)mmap(nullptr, total, PROT_READ | PROT_WRITE, MAP_PRIVATE | MAP_ANONYMOUS, -1, 0);
    if (base == MAP_FAILED) return nullptr;
    mprotect(base, page, PROT_NONE);
    mprotect(base + page + body, page, PROT_NONE);
    uint8_t* p = base + page + (body - sz);
    memset(base + page, 0xCD, body - sz);
    std::lock_guard<std::mutex> lk(alloc_mu);
    allocs.push_back({p, Alloc{base, total}});
    return p;
}
void dev_free(void* p)
{
    if (!p) return;
    std::lock_guard<std::mutex> lk(alloc_mu);
    for (size_t i = 0; i < allocs.size(); ++i)
        if (allocs[i].first == p) {
            munmap(allocs[i].second.base, allocs[i].second.total);
            allocs.erase(allocs.begin() + i);
            return;
        }
}
}  // namespace emu

namespace emu {
static void on_segv(int, siginfo_t* si, void*)
{
    const uint8_t* a = (const uint8_t*)si->si_addr;
    fprintf(stderr, "emu: SIGSEGV at address %p", (void*)a);
    if (G) fprintf(stderr, " in block (%u,%u) thread %d", G->block.x, G->block.y, G->f[G->current].linear);
    fprintf(stderr, "\n");
    for (size_t i = 0; i < allocs.size(); ++i) {
        const uint8_t* b = (const uint8_t*)allocs[i].second.base;
        if (a >= b && a < b + allocs[i].second.total)
            fprintf(stderr, "  inside the guard region of allocation #%zu (user pointer %p, offset from it %ld)\n", i, allocs[i].first,
                    (long)(a - (const uint8_t*)allocs[i].first));
    }
    void* bt[32];
    const int n = backtrace(bt, 32);
    backtrace_symbols_fd(bt, n, 2);
    _exit(139);
}
struct Install { Install() {
    static uint8_t altstack[65536];
    stack_t ss{}; ss.ss_sp = altstack; ss.ss_size = sizeof(altstack); sigaltstack(&ss, nullptr);
    struct sigaction sa{}; sa.sa_sigaction = on_segv; sa.sa_flags = SA_SIGINFO | SA_ONSTACK; sigaction(SIGSEGV, &sa, nullptr); } } install;
}
// the instruction-rate measurement has no meaning on the host
extern "C" int spmm_measure_peak(int, double*) { return 2; /* SPMM_E_UNSUPPORTED */ }
extern "C" void* emu_alloc(size_t bytes) { return emu::dev_alloc(bytes); }
extern "C" void emu_free(void* p) { emu::dev_free(p); }
