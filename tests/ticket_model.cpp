// Host model of the hand-off that the one-launch prediction kernel uses between the workgroups of a frame (the
// last of SLICES groups to finish its fully connected outputs runs the heads of Sec. 3.2).  Threads stand for
// wavefronts, WAVES of them make a group with a barrier of its own.  Built with -fsanitize=thread by
// tests/test_abi_cpu.py: the sanitizer checks that every read of h by the last group is ordered after every
// write of it, which is what the kernel gets from "each wavefront waits for the acknowledgement of its stores,
// barrier, device-scope ticket".  The model states that guarantee as release/acquire on the ticket; with the
// argument "relaxed" the ordering is left out on purpose and the sanitizer must report the race (the harness
// checks both).  Plain floats for h, so that the sanitizer tracks them.
//
//   ticket_model [relaxed] -> exit 0 and "ok <launches>" when every launch ended with one finisher per frame that
//   saw all outputs, and all tickets back at zero.
#include <atomic>
#include <cstdio>
#include <cstring>
#include <pthread.h>
#include <thread>
#include <vector>

namespace {
constexpr int FRAMES = 3, SLICES = 4, WAVES = 2, FC = 32, LAUNCHES = 200;
constexpr int ROWS = FC / (SLICES * WAVES);       // outputs per wavefront

float h[FRAMES][FC];
std::atomic<int> ticket[FRAMES];
std::atomic<int> finishers[FRAMES];
std::atomic<int> bad{0};
bool relaxed_ticket = false;

struct Group {
    pthread_barrier_t bar;
    int last = 0;
};

void wavefront(Group *g, int launch, int frame, int slice, int wave) {
    for (int r = 0; r < ROWS; ++r) {
        const int o = (slice * WAVES + wave) * ROWS + r;
        h[frame][o] = float(launch * 1000 + frame * 100 + o);       // the store of an fc output
    }
    // kernel: s_waitcnt vmcnt(0) (own stores acknowledged), then the barrier of the group
    pthread_barrier_wait(&g->bar);
    if (wave == 0) {
        const auto order = relaxed_ticket ? std::memory_order_relaxed : std::memory_order_acq_rel;
        const int t = ticket[frame].fetch_add(1, order);
        g->last = t == SLICES - 1;
        if (g->last) ticket[frame].store(0, std::memory_order_relaxed);      // for the next launch
    }
    pthread_barrier_wait(&g->bar);
    if (!g->last) return;
    if (wave == 0) finishers[frame].fetch_add(1, std::memory_order_relaxed);
    // the heads: every wavefront of the finishing group reads outputs written by all groups
    for (int o = wave; o < FC; o += WAVES)
        if (h[frame][o] != float(launch * 1000 + frame * 100 + o)) bad.fetch_add(1, std::memory_order_relaxed);
}
}  // namespace

int main(int argc, char **argv) {
    relaxed_ticket = argc > 1 && !std::strcmp(argv[1], "relaxed");
    for (int launch = 0; launch < LAUNCHES; ++launch) {
        std::vector<Group> groups(FRAMES * SLICES);
        for (auto &g : groups) pthread_barrier_init(&g.bar, nullptr, WAVES);
        for (int f = 0; f < FRAMES; ++f) finishers[f].store(0);
        std::vector<std::thread> th;
        for (int f = 0; f < FRAMES; ++f)
            for (int s = 0; s < SLICES; ++s)
                for (int w = 0; w < WAVES; ++w) th.emplace_back(wavefront, &groups[f * SLICES + s], launch, f, s, w);
        for (auto &t : th) t.join();       // the end of the launch: stream order puts the next one after it
        for (auto &g : groups) pthread_barrier_destroy(&g.bar);
        for (int f = 0; f < FRAMES; ++f) {
            if (finishers[f].load() != 1) { std::printf("launch %d frame %d: %d finishers\n", launch, f, finishers[f].load()); return 1; }
            if (ticket[f].load() != 0) { std::printf("launch %d frame %d: ticket left at %d\n", launch, f, ticket[f].load()); return 1; }
        }
        if (bad.load()) { std::printf("launch %d: %d stale outputs read\n", launch, bad.load()); return 1; }
    }
    std::printf("ok %d\n", LAUNCHES);
    return 0;
}
