// CPU-only stress of the task state machine (paper_2602_16603_amd/csrc/task_core.h) against a
// stand-in device whose operators just take time.  Built with -fsanitize=thread by
// tests/test_task_core_tsan.py: an executor thread advances tasks, a scheduler thread raises
// preempt signals at random moments, waits for the acknowledgement and resumes, and a third thread
// polls the cursor -- the calls the C ABI allows to run concurrently (FlowPrefill Section 5.1: the
// scheduler signals, the worker acknowledges at an operator boundary).  Exit code 0 = every
// invariant held; ThreadSanitizer adds its own report and exit code on a data race.
#include <atomic>
#include <chrono>
#include <cstdio>
#include <cstdlib>
#include <random>
#include <thread>
#include <vector>

#include "../../paper_2602_16603_amd/csrc/task_core.h"

using Clock = std::chrono::steady_clock;

#define CHECK(cond)                                                          \
  do {                                                                       \
    if (!(cond)) {                                                           \
      std::fprintf(stderr, "CHECK failed: %s (line %d)\n", #cond, __LINE__); \
      std::exit(1);                                                          \
    }                                                                        \
  } while (0)

// An in-order "stream": an operator starts when its predecessor ends and lasts op_us microseconds.
// Only the thread inside advance touches it (as with the real backend).
struct FakeDevice : fp::OpBackend {
  int32_t total, launch_ahead;
  std::vector<int> runs;                 // how often each operator was enqueued
  std::vector<Clock::time_point> end_of; // completion time of each operator
  Clock::time_point free_at = Clock::now();
  Clock::time_point mark_at[fp::kMarkRing];
  int32_t mark_op[fp::kMarkRing];
  int32_t last = -1, calls = 0, first_of_call = 0;
  std::mt19937 rng;
  FakeDevice(int32_t n, int32_t ahead, uint32_t seed) : total(n), launch_ahead(ahead), runs(n, 0), end_of(n), rng(seed) {}

  std::vector<Clock::time_point> work_ends;   // completion times of this call's operators with device work
  void begin_call() override { ++calls; first_of_call = last + 1; work_ends.clear(); }
  int launch(int32_t index, bool* launched) override {
    CHECK(index == last + 1);                       // in order, none skipped, none repeated
    CHECK(index < total);
    *launched = index % 9 != 7;                     // one operator per layer has no device work
    if (*launched) {
      // Launch-ahead bound: of this call's operators with device work, all but the last
      // launch_ahead must be complete by now.
      if (launch_ahead > 0 && (int32_t)work_ends.size() >= launch_ahead)
        CHECK(work_ends[work_ends.size() - launch_ahead] <= Clock::now());
      const auto start = std::max(Clock::now(), free_at);
      free_at = start + std::chrono::microseconds(20 + rng() % 200);
      work_ends.push_back(free_at);
    }
    end_of[index] = free_at;
    runs[index]++;
    last = index;
    return 0;
  }
  int mark(int slot) override { mark_at[slot] = free_at; mark_op[slot] = last; return 0; }
  int wait_mark(int slot) override { std::this_thread::sleep_until(mark_at[slot]); return 0; }
  int drain() override { std::this_thread::sleep_until(free_at); return 0; }
  bool drained() const { return free_at <= Clock::now(); }
};

int main(int argc, char** argv) {
  const int n_tasks = argc > 1 ? std::atoi(argv[1]) : 40;
  const uint32_t masks[4] = {0x1FF, 0x15A, 0x100, 0x0};
  long parks = 0, races_with_done = 0, idle_parks = 0;
  for (int it = 0; it < n_tasks; ++it) {
    const int32_t layers = 2 + it % 3, total = layers * 9;
    const uint32_t mask = masks[it % 4];
    const int32_t ahead = it % 3;                   // 0 = unbounded, 1, 2
    fp::TaskCore core(total, 9, mask);
    FakeDevice dev(total, ahead, 1234u + it);
    CHECK(core.set_launch_ahead(ahead) == fp::kTaskOk);
    std::atomic<bool> finished{false};
    std::atomic<int> parked_seen{0};

    std::thread executor([&] {
      std::mt19937 rng(99u + it);
      for (;;) {
        int32_t done = -1;
        const int32_t want = 1 + rng() % 12;
        const int32_t before = core.cursor();
        const int r = core.advance(dev, want, &done);
        if (r == fp::kTaskErrState) {               // parked by the scheduler while idle: wait for the resume
          std::this_thread::yield();
          continue;
        }
        CHECK(r >= 0);
        CHECK(done >= 0 && done <= want);
        CHECK(core.cursor() == before + done);
        CHECK(dev.drained());                       // every return leaves the device quiescent
        if (r == fp::kTaskPreempted) {
          const int32_t c = core.cursor();
          // Parked inside a call (done < want and operators remain): only at an enabled boundary.
          if (done < want && c > 0 && c < total) CHECK((mask >> ((c - 1) % 9)) & 1u);
          parked_seen.fetch_add(1);
        }
        if (r == fp::kTaskDone) break;
        if (rng() % 3 == 0) std::this_thread::sleep_for(std::chrono::microseconds(rng() % 400));   // idle between calls
      }
      finished.store(true);
    });

    std::thread poller([&] {
      int32_t seen = 0;
      while (!finished.load()) {
        const int32_t c = core.cursor();
        CHECK(c >= seen && c <= total);             // monotone, in range
        seen = c;
      }
    });

    std::thread scheduler([&] {
      std::mt19937 rng(7u + it);
      while (!finished.load()) {
        std::this_thread::sleep_for(std::chrono::microseconds(rng() % 1500));
        const int s = core.preempt_signal();
        if (s == fp::kTaskDone) break;
        if (s == fp::kTaskErrState) continue;       // still parked from the last round (cannot happen here)
        int r = s;
        if (s == fp::kTaskOk) r = core.preempt_wait();
        else idle_parks++;
        if (r == fp::kTaskDone) { races_with_done++; break; }
        CHECK(r == fp::kTaskPreempted);
        CHECK(core.state() == fp::TaskState::Parked);
        const int32_t c = core.cursor();
        std::this_thread::sleep_for(std::chrono::microseconds(rng() % 300));   // the other request runs
        CHECK(core.cursor() == c);                  // a parked task does not move
        CHECK(core.advance(dev, 1, nullptr) == fp::kTaskErrState);   // a parked task refuses to advance (the device is not touched)
        parks++;
        CHECK(core.resume() == fp::kTaskOk);
      }
    });

    executor.join();
    scheduler.join();
    poller.join();
    CHECK(core.cursor() == total);
    CHECK(core.state() == fp::TaskState::Done);
    for (int32_t i = 0; i < total; ++i) CHECK(dev.runs[i] == 1);   // resume continues, never repeats
    CHECK(core.preempt_signal() == fp::kTaskDone);
    CHECK(core.resume() == fp::kTaskErrState);
  }
  std::printf("task_core_race: %d tasks, %ld parks (%ld while idle), %ld signals raced with completion: OK\n",
              n_tasks, parks, idle_parks, races_with_done);
  return 0;
}
