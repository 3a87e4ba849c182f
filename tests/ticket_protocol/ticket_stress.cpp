// CPU stress of the ticket protocol that merges the partial results of several work-groups in
// the short-chunk kernel (decode_body in csrc/evl_kernels.hip), with host threads standing in
// for work-groups and C++ atomics for the device-scope ones.  Protocol per launch and per group
// of n pieces: every piece publishes its partial result, then takes a ticket from a counter;
// the holder of the last ticket -- and nobody else -- reads all partial results, writes the
// output and puts the counter back to zero for the next launch.  Checked over many rounds with
// random arrival orders: exactly one merger per round, the merger sees every piece of THIS
// round, the counter is zero between rounds.  (What this cannot check is the GPU's memory
// model; it checks that the counting logic has no hole.)  Test infrastructure only.
#include <atomic>
#include <cstdio>
#include <cstdlib>
#include <random>
#include <thread>
#include <vector>

int main(int argc, char **argv) {
    const int pieces = argc > 1 ? atoi(argv[1]) : 14, rounds = argc > 2 ? atoi(argv[2]) : 20000;
    std::atomic<int> counter{0};
    std::vector<std::atomic<long>> partial(pieces);
    std::atomic<long> out{-1};
    std::atomic<int> mergers{0}, start{0}, done{0};
    std::atomic<bool> failed{false};
    auto piece = [&](int me) {
        std::mt19937 rng(1234 + me);
        for (int r = 0; r < rounds && !failed; ++r) {
            while (start.load(std::memory_order_acquire) <= r) std::this_thread::yield();   // the launch
            for (int spin = (int)(rng() % 200); spin > 0; --spin) std::atomic_signal_fence(std::memory_order_seq_cst);
            partial[me].store((long)r * 1000 + me, std::memory_order_relaxed);    // publish the partial result
            const int ticket = counter.fetch_add(1, std::memory_order_acq_rel);   // ... then take a ticket
            if (ticket == pieces - 1) {                                           // last one in: merge
                mergers.fetch_add(1);
                long sum = 0;
                for (int p = 0; p < pieces; ++p) {
                    const long v = partial[p].load(std::memory_order_relaxed);
                    if (v / 1000 != r) failed = true;                             // a piece of another round
                    sum += v;
                }
                out.store(sum);
                counter.store(0, std::memory_order_release);                      // ready for the next launch
            }
            done.fetch_add(1, std::memory_order_release);
        }
    };
    std::vector<std::thread> ts;
    for (int p = 0; p < pieces; ++p) ts.emplace_back(piece, p);
    for (int r = 0; r < rounds && !failed; ++r) {
        if (counter.load() != 0) { failed = true; break; }                         // zero between launches
        mergers = 0;
        done = 0;
        start.store(r + 1, std::memory_order_release);
        while (done.load(std::memory_order_acquire) < pieces) std::this_thread::yield();   // the launch has drained
        long want = 0;
        for (int p = 0; p < pieces; ++p) want += (long)r * 1000 + p;
        if (mergers.load() != 1 || out.load() != want || counter.load() != 0) failed = true;
    }
    start.store(rounds + 1);
    failed ? (void)start.store(1 << 30) : (void)0;
    for (auto &t : ts) t.join();
    printf(failed ? "FAILED\n" : "ok: %d pieces, %d rounds, one merger per round\n", pieces, rounds);
    return failed ? 1 : 0;
}
