// Host-only exercise of the library's CPU-side code for the sanitizer builds (AddressSanitizer +
// UndefinedBehaviorSanitizer, and ThreadSanitizer): the host-CPU step and reduction, the chunk planner,
// the thread pool with memory and file pieces (direct-I/O bounce path included), the parked stage
// threads, and a model of the pinned ring's three-actor choreography (gather thread, issuing thread,
// scatter thread advancing three counters under one mutex) built from the same primitives.  The oracle's
// C file is compiled in as well and called on the same inputs.  Exit status 0 = all checks passed; the
// sanitizers report anything else on stderr.
#include <fcntl.h>
#include <unistd.h>

#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "zi_checks.h"
#include "zi_io_pool.h"
#include "zi_plan.h"

#include "zi_oracle.h"

namespace zi {
namespace host {
static thread_local char g_err[256];
zi_status fail(zi_status st, const char* fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return st;
}
const char* last_error() { return g_err; }
}  // namespace host
}  // namespace zi

using namespace zi::host;

#define CHECK(cond)                                                          \
    do {                                                                     \
        if (!(cond)) {                                                       \
            fprintf(stderr, "CHECK failed: %s (line %d)\n", #cond, __LINE__); \
            return 1;                                                        \
        }                                                                    \
    } while (0)

static uint32_t lcg(uint32_t& s) { return s = s * 1664525u + 1013904223u; }

static int host_step_checks()
{
    uint32_t seed = 12345;
    for (int dt = 0; dt < 2; ++dt)
        for (int64_t n : {0, 1, 7, 8, 9, 1000, (1 << 18) + 3, 600001}) {
            std::vector<float> p((size_t)n), m((size_t)n), v((size_t)n), p2, m2, v2;
            std::vector<uint16_t> g((size_t)n), lp((size_t)n, 0), lp2((size_t)n, 0);
            for (int64_t i = 0; i < n; ++i) {
                p[(size_t)i] = ((int)(lcg(seed) >> 8) - (1 << 23)) * 1e-8f;
                m[(size_t)i] = ((int)(lcg(seed) >> 8) - (1 << 23)) * 1e-11f;
                v[(size_t)i] = (lcg(seed) >> 8) * 1e-13f;
                g[(size_t)i] = (uint16_t)((dt == 0 ? 0x3A00 : 0x1400) + (lcg(seed) >> 24));
            }
            p2 = p; m2 = m; v2 = v;
            zi_tensor t{p.data(), m.data(), v.data(), g.data(), lp.data(), n};
            zi_adamw_config cfg{1e-3f, 0.9f, 0.999f, 1e-8f, 0.01f, 10, 4.0f, 0.01f, ZI_MODE_ADAMW};
            zi_norm_result nr{};
            CHECK(zi_host_grad_norm(&t, 1, (zi_lp_dtype)dt, 4.0f, &nr, 4) == ZI_OK);
            CHECK(zi_host_adamw_step(&t, 1, (zi_lp_dtype)dt, &cfg, &nr, 4) == ZI_OK);
            // the oracle on the same inputs
            zio_config oc;
            memset(&oc, 0, sizeof oc);
            oc.lr = 1e-3f; oc.beta1 = 0.9f; oc.beta2 = 0.999f; oc.eps = 1e-8f; oc.weight_decay = 0.01f;
            oc.step = 10; oc.loss_scale = 4.0f; oc.max_grad_norm = 0.01f; oc.mode = 0;
            zio_sumsq_state acc;
            zio_sumsq_init(&acc);
            zio_sumsq_accumulate(&acc, g.data(), n, dt);
            const double ss = zio_sumsq_value(&acc);
            const uint32_t fl = acc.found_inf;
            CHECK(fl == 0 && nr.found_inf == 0);
            CHECK(zio_adamw(p2.data(), m2.data(), v2.data(), g.data(), lp2.data(), n, dt, &oc, 1, ss, fl) == 0);
            CHECK(n == 0 || memcmp(p.data(), p2.data(), (size_t)n * 4) == 0);
            CHECK(n == 0 || memcmp(v.data(), v2.data(), (size_t)n * 4) == 0);
            CHECK(n == 0 || memcmp(lp.data(), lp2.data(), (size_t)n * 2) == 0);
        }
    return 0;
}

static int plan_checks()
{
    std::vector<Segment> segs;
    int64_t uses = 0;
    std::vector<int64_t> numel;
    uint32_t seed = 7;
    for (int round = 0; round < 50; ++round) {
        numel.clear();
        const int k = (int)(lcg(seed) % 60);
        for (int i = 0; i < k; ++i) numel.push_back((int64_t)(lcg(seed) % 3 == 0 ? lcg(seed) % 50000 : lcg(seed) % 200));
        plan_chunks(numel.data(), k, 4096, segs, uses);
        int64_t total = 0, want = 0;
        for (const Segment& s : segs) {
            CHECK(s.tensor >= 0 && s.tensor < k && s.count > 0 && s.slot_use >= 0 && s.slot_use < uses);
            CHECK(s.slot_offset + s.count <= 4096);
            total += s.count;
        }
        for (int64_t x : numel) want += x;
        CHECK(total == want);
    }
    return 0;
}

static int pool_checks()
{
    const size_t bytes = 3 * kCopyPieceBytes + 12345 - 12345 % 4096;
    std::vector<char> a(bytes), b(bytes, 0), c(bytes, 0);
    for (size_t i = 0; i < bytes; ++i) a[i] = (char)(i * 131 + 7);
    TaskPool pool(5);
    std::vector<Piece> pieces;
    for (size_t o = 0; o < bytes; o += 1 << 20) {
        const size_t nb = bytes - o < (1u << 20) ? bytes - o : (1u << 20);
        pieces.push_back({0, b.data() + o, a.data() + o, -1, 0, nb, nb, false});
    }
    CHECK(run_pieces(pool, pieces) == 0);
    CHECK(memcmp(a.data(), b.data(), bytes) == 0);
    // through a file, with and without the aligned bounce buffer
    char path[] = "/tmp/zi_host_sanity_XXXXXX";
    const int fd = mkstemp(path);
    CHECK(fd >= 0);
    for (int bounce = 0; bounce < 2; ++bounce) {
        pieces.clear();
        for (size_t o = 0; o < bytes; o += kCopyPieceBytes) {
            const size_t nb = bytes - o < kCopyPieceBytes ? bytes - o : kCopyPieceBytes;
            pieces.push_back({2, a.data() + o, nullptr, fd, (int64_t)o, nb, nb, bounce != 0});
        }
        CHECK(run_pieces(pool, pieces) == 0);
        pieces.clear();
        std::fill(c.begin(), c.end(), 0);
        for (size_t o = 0; o < bytes; o += kCopyPieceBytes) {
            const size_t nb = bytes - o < kCopyPieceBytes ? bytes - o : kCopyPieceBytes;
            pieces.push_back({1, c.data() + o, nullptr, fd, (int64_t)o, nb, nb, bounce != 0});
        }
        CHECK(run_pieces(pool, pieces) == 0);
        CHECK(memcmp(a.data(), c.data(), bytes) == 0);
    }
    // a read beyond the end of the file is an error code, not a crash
    pieces.clear();
    pieces.push_back({1, c.data(), nullptr, fd, (int64_t)bytes, 4096, 4096, false});
    CHECK(run_pieces(pool, pieces) == EIO);
    pieces.clear();
    pieces.push_back({1, c.data(), nullptr, -1, 0, 4096, 4096, false});
    CHECK(run_pieces(pool, pieces) == EBADF);
    close(fd);
    unlink(path);
    return 0;
}

// The ring's choreography in miniature: a "device" that is just a buffer, ring slots, a gather stage
// that fills slot u mod H once the scatter stage has emptied its previous contents, the caller's thread
// that "updates" a gathered slot, and a scatter stage that writes it back.
struct RingModel {
    static constexpr int H = 3;
    int64_t n_uses;
    size_t chunk;
    std::vector<float>* state;
    std::vector<float> ring[H];
    TaskPool* pool_in;
    TaskPool* pool_out;
    std::vector<Piece> pin, pout;
    std::mutex mu;
    std::condition_variable cv;
    int64_t gathered = 0, issued = 0, scattered = 0;
    bool abort = false;

    static void gather(void* ctx)
    {
        RingModel& r = *static_cast<RingModel*>(ctx);
        for (int64_t u = 0; u < r.n_uses; ++u) {
            {
                std::unique_lock<std::mutex> lk(r.mu);
                r.cv.wait(lk, [&] { return r.abort || r.scattered >= u - H + 1; });
                if (r.abort) return;
            }
            r.pin.clear();
            r.pin.push_back({0, (char*)r.ring[u % H].data(), (const char*)(r.state->data() + (size_t)u * r.chunk), -1, 0,
                             r.chunk * 4, r.chunk * 4, false});
            (void)run_pieces(*r.pool_in, r.pin);
            {
                std::lock_guard<std::mutex> lk(r.mu);
                r.gathered = u + 1;
            }
            r.cv.notify_all();
        }
    }
    static void scatter(void* ctx)
    {
        RingModel& r = *static_cast<RingModel*>(ctx);
        for (int64_t u = 0; u < r.n_uses; ++u) {
            {
                std::unique_lock<std::mutex> lk(r.mu);
                r.cv.wait(lk, [&] { return r.abort || r.issued > u; });
                if (r.abort) return;
            }
            r.pout.clear();
            r.pout.push_back({0, (char*)(r.state->data() + (size_t)u * r.chunk), (const char*)r.ring[u % H].data(), -1, 0,
                              r.chunk * 4, r.chunk * 4, false});
            (void)run_pieces(*r.pool_out, r.pout);
            {
                std::lock_guard<std::mutex> lk(r.mu);
                r.scattered = u + 1;
            }
            r.cv.notify_all();
        }
    }
};

static int ring_checks()
{
    TaskPool pin(3), pout(3);
    StageThread sin, sout;
    for (int round = 0; round < 3; ++round) {          // the parked threads serve several "calls"
        RingModel r;
        r.n_uses = 40;
        r.chunk = 5000;
        std::vector<float> state((size_t)r.n_uses * r.chunk);
        for (size_t i = 0; i < state.size(); ++i) state[i] = (float)i;
        r.state = &state;
        for (auto& s : r.ring) s.assign(r.chunk, 0.0f);
        r.pool_in = &pin;
        r.pool_out = &pout;
        sin.start(&RingModel::gather, &r);
        sout.start(&RingModel::scatter, &r);
        for (int64_t u = 0; u < r.n_uses; ++u) {
            {
                std::unique_lock<std::mutex> lk(r.mu);
                r.cv.wait(lk, [&] { return r.gathered > u; });
            }
            for (float& x : r.ring[u % RingModel::H]) x += 1.0f;      // the "update"
            {
                std::lock_guard<std::mutex> lk(r.mu);
                r.issued = u + 1;
            }
            r.cv.notify_all();
        }
        sin.wait();
        sout.wait();
        for (size_t i = 0; i < state.size(); ++i) CHECK(state[i] == (float)i + 1.0f);
    }
    return 0;
}

int main()
{
    if (!host_step_supported()) {
        printf("skipped: no AVX2/FMA/F16C\n");
        return 0;
    }
    if (int rc = host_step_checks()) return rc;
    if (int rc = plan_checks()) return rc;
    if (int rc = pool_checks()) return rc;
    if (int rc = ring_checks()) return rc;
    printf("host sanity ok\n");
    return 0;
}
