// Runtime of the CPU emulation: a pool of 256 OS threads plays the threads of one block;
// blocks of a launch run one after another.
#include <hip/hip_runtime.h>

#include <chrono>
#include <condition_variable>
#include <execinfo.h>
#include <mutex>
#include <sched.h>
#include <signal.h>
#include <sys/mman.h>
#include <thread>
#include <unistd.h>
#include <vector>

thread_local dim3 threadIdx, blockIdx;
dim3 blockDim, gridDim;
thread_local const char* emu_where = "";
thread_local int emu_line = 0;
alignas(64) static char g_lds[160 * 1024];
char* emu_dyn_lds = g_lds;

constexpr int MAXT = 256;
static thread_local int t_id = -1;   // index in the pool, -1: host thread
static const char* g_where[MAXT];
static int g_wline[MAXT];
static int g_block = 0;
static const char* g_kernel = "";

static void dump_all(const char* why) {
    fprintf(stderr, "\n[emu] %s; block %d of %u, blockDim %u\n", why, g_block, gridDim.x, blockDim.x);
    for (unsigned t = 0; t < blockDim.x && t < MAXT; ++t)
        if (t < 8 || t % 64 == 0 || t % 64 == 63 || g_wline[t] != g_wline[0])
            fprintf(stderr, "  thread %3u last at %s:%d\n", t, g_where[t] ? g_where[t] : "?", g_wline[t]);
    fflush(stderr);
}
static void note() {
    if (t_id >= 0) { g_where[t_id] = emu_where; g_wline[t_id] = emu_line; }
}

struct Barrier {
    std::mutex m;
    std::condition_variable cv;
    int count = 0, n = 0;
    uint64_t gen = 0;
    void init(int n_) { n = n_; count = 0; }
    void wait(const char* what) {
        note();
        std::unique_lock<std::mutex> lk(m);
        const uint64_t g = gen;
        if (++count >= n) { count = 0; ++gen; cv.notify_all(); return; }
        if (what[0] == 's' && what[1] == 't') { cv.wait(lk, [&] { return gen != g; }); return; }   // idle pool
        // the launching thread waits for the whole launch: long for a large case, and a hang inside
        // it is reported by the workers' own waits
        if (what[0] == 'd' && what[1] == 'o') { cv.wait(lk, [&] { return gen != g; }); return; }
        // a wait that outlasts the limit is taken for a deadlock; the end-of-launch wait of a large
        // case legitimately takes long (EMU_WAIT_SECONDS raises the limit)
        static const int limit = getenv("EMU_WAIT_SECONDS") ? atoi(getenv("EMU_WAIT_SECONDS")) : 60;
        if (!cv.wait_for(lk, std::chrono::seconds(limit), [&] { return gen != g; })) {
            fprintf(stderr, "[emu] barrier '%s' timed out: %d of %d arrived (thread %d)\n", what, count, n, t_id);
            dump_all("deadlock");
            abort();
        }
    }
    // a thread that leaves the kernel no longer takes part in __syncthreads
    void leave() {
        std::unique_lock<std::mutex> lk(m);
        --n;
        if (n > 0 && count >= n) { count = 0; ++gen; cv.notify_all(); }
    }
};

static Barrier &b_start = *new Barrier, &b_done = *new Barrier, &b_blk = *new Barrier, &b_sync = *new Barrier;
static Barrier* const b_wave = new Barrier[4];   // never destroyed: idle workers sleep on them at exit
static std::function<void()> g_body;
static int g_nthreads = 0;
static std::vector<std::thread>& g_pool = *new std::vector<std::thread>;
static std::atomic<long long> g_clock{0};

static void on_segv(int sig, siginfo_t* si, void*) {
    fprintf(stderr, "\n[emu] signal %d at address %p: block %u thread %u (pool %d), last collective %s:%d\n", sig,
            si->si_addr, blockIdx.x, threadIdx.x, t_id, emu_where, emu_line);
    void* bt[48];
    const int n = backtrace(bt, 48);
    backtrace_symbols_fd(bt, n, 2);
    _exit(139);
}

static void worker(int id) {
    t_id = id;
    for (;;) {
        b_start.wait("start");
        if (id < g_nthreads) {
            for (unsigned blk = 0; blk < gridDim.x * gridDim.y * gridDim.z; ++blk) {
                blockIdx = dim3(blk % gridDim.x, (blk / gridDim.x) % gridDim.y, blk / (gridDim.x * gridDim.y));
                threadIdx = dim3(id % blockDim.x, (id / blockDim.x) % blockDim.y, id / (blockDim.x * blockDim.y));
                if (id == 0) { g_block = (int)blk; b_sync.init(g_nthreads); }
                b_blk.wait("block begin");
                g_body();
                b_sync.leave();
                b_blk.wait("block end");
            }
        }
        b_done.wait("done");
    }
}

void emu_launch(const std::function<void()>& body, dim3 grid, dim3 block, size_t shmem, bool coop) {
    static bool once = false;
    if (!once) {
        once = true;
        struct sigaction sa;
        memset(&sa, 0, sizeof sa);
        sa.sa_sigaction = on_segv;
        sa.sa_flags = SA_SIGINFO;
        sigaction(SIGSEGV, &sa, nullptr);
        sigaction(SIGBUS, &sa, nullptr);
        b_start.init(MAXT + 1);
        b_done.init(MAXT + 1);
        for (int i = 0; i < MAXT; ++i) g_pool.emplace_back(worker, i);
        for (auto& t : g_pool) t.detach();
    }
    const int nt = (int)(block.x * block.y * block.z);
    if (nt > MAXT || nt % 64) { fprintf(stderr, "[emu] unsupported block size %d\n", nt); abort(); }
    if (shmem > sizeof g_lds) { fprintf(stderr, "[emu] dynamic LDS too large\n"); abort(); }
    if (coop && grid.x * grid.y * grid.z != 1) { fprintf(stderr, "[emu] cooperative launches: one block only\n"); abort(); }
    if (grid.x * grid.y * grid.z == 0) return;
    g_body = body;
    gridDim = grid;
    blockDim = block;
    g_nthreads = nt;
    b_blk.init(nt);
    b_sync.init(nt);
    for (int w = 0; w < 4; ++w) b_wave[w].init(64);
    b_start.wait("start");
    b_done.wait("done");
}

void emu_syncthreads() { b_sync.wait("__syncthreads"); }
void emu_yield() { sched_yield(); }
long long emu_clock() { return ++g_clock; }

// ---- pairwise exchange for __shfl_xor ----
struct Slot {
    std::atomic<uint64_t> seq[8];
    uint64_t cnt[8];
    uint32_t val[8][4];
};
static Slot g_slot[MAXT];

uint32_t emu_shfl_xor32(uint32_t v, int mask) {
    // one exchange channel per mask: the powers of two, and 7 / 15 (the mirrored half row / row of the
    // DPP permutations, which are the exchanges i <-> i ^ 7 and i <-> i ^ 15)
    const bool pow2 = mask > 0 && mask < 64 && !(mask & (mask - 1));
    if (!pow2 && mask != 7 && mask != 15) { fprintf(stderr, "[emu] shfl_xor mask %d\n", mask); abort(); }
    const int bit = pow2 ? __builtin_ctz(mask) : mask == 7 ? 6 : 7, me = t_id, other = me ^ mask;
    Slot& a = g_slot[me];
    Slot& b = g_slot[other];
    const uint64_t k = a.cnt[bit]++;
    a.val[bit][k & 3] = v;
    a.seq[bit].store(k + 1, std::memory_order_release);
    note();
    long spins = 0;
    while (b.seq[bit].load(std::memory_order_acquire) < k + 1) {
        sched_yield();
        if (++spins > 20000000) {
            fprintf(stderr, "[emu] shfl_xor(%d): lane %d waits for lane %d that never came (%s:%d)\n", mask, me, other,
                    emu_where, emu_line);
            dump_all("divergent shuffle");
            abort();
        }
    }
    return b.val[bit][k & 3];
}

static uint32_t g_xch[MAXT];
uint32_t emu_shfl_down32(uint32_t v, int delta) {
    const int me = t_id, w = me >> 6, lane = me & 63;
    g_xch[me] = v;
    b_wave[w].wait("shfl_down");
    const uint32_t r = lane + delta < 64 ? g_xch[me + delta] : v;
    b_wave[w].wait("shfl_down");
    return r;
}

uint32_t emu_shfl_idx32(uint32_t v, int src) {
    const int me = t_id, w = me >> 6;
    g_xch[me] = v;
    b_wave[w].wait("shfl");
    const uint32_t r = g_xch[(w << 6) + (src & 63)];
    b_wave[w].wait("shfl");
    return r;
}

int emu_all(int pred) {
    const int me = t_id, w = me >> 6;
    g_xch[me] = pred ? 1 : 0;
    b_wave[w].wait("all");
    int r = 1;
    for (int i = 0; i < 64; ++i) r &= (int)g_xch[(w << 6) + i];
    b_wave[w].wait("all");
    return r;
}

static uint16_t g_a[MAXT][8], g_b[MAXT][8];
static inline float bf(uint16_t x) { uint32_t u = (uint32_t)x << 16; float f; memcpy(&f, &u, 4); return f; }
void emu_mfma_16x16x32_bf16(const uint16_t a[8], const uint16_t b[8], float c[4]) {
    const int me = t_id, w = me >> 6, lane = me & 63, base = w * 64;
    memcpy(g_a[me], a, 16);
    memcpy(g_b[me], b, 16);
    b_wave[w].wait("mfma");
    const int col = lane & 15;
    for (int i = 0; i < 4; ++i) {
        const int row = 4 * (lane >> 4) + i;
        float acc = 0.f;
        for (int k = 0; k < 32; ++k)
            acc += bf(g_a[base + row + 16 * (k >> 3)][k & 7]) * bf(g_b[base + col + 16 * (k >> 3)][k & 7]);
        c[i] += acc;
    }
    b_wave[w].wait("mfma");
}

// Arena with inaccessible pages on both sides; the usable range ends right at the upper guard.
extern "C" void* emu_alloc(size_t n, int fill) {
    const size_t pg = 4096, body = (n + 255) / 256 * 256, span = (body + pg - 1) / pg * pg;
    char* p = (char*)mmap(nullptr, span + 2 * pg, PROT_READ | PROT_WRITE, MAP_PRIVATE | MAP_ANONYMOUS, -1, 0);
    if (p == MAP_FAILED) return nullptr;
    mprotect(p, pg, PROT_NONE);
    mprotect(p + pg + span, pg, PROT_NONE);
    char* base = p + pg + (span - body);
    memset(p + pg, fill, span);
    return base;
}
