// Host-side state machine of one execution task: operator cursor, bounded launch-ahead and the
// cooperative preemption gate (FlowPrefill Section 5.1: the runtime looks at a signal between
// operators; if it is set, the work in flight finishes, the signal is cleared, an acknowledgement is
// sent and the task is suspended with its state in place.  Section 4: a suspended task keeps its
// state until it is resumed).
//
// This header is plain C++17 with no GPU dependency: everything the state machine needs from the
// device sits behind OpBackend, so that the locking and signalling can be built for the CPU with a
// stand-in backend and run under ThreadSanitizer.
#pragma once
#include <atomic>
#include <condition_variable>
#include <cstdint>
#include <mutex>

namespace fp {

enum class TaskState { Idle, Running, Parked, Done };

constexpr int kMarkRing = 8;   // completion markers in flight at most (bounds launch_ahead)

// Result codes; the values are those of fp_status in the C header.
enum { kTaskOk = 0, kTaskDone = 1, kTaskPreempted = 2, kTaskErrInvalid = -1, kTaskErrState = -3, kTaskErrDevice = -4 };

// What the state machine asks of the device side.  Every call returns 0 or a negative code (the
// backend records its own error text).  Only the thread inside TaskCore::advance calls these.
struct OpBackend {
  virtual ~OpBackend() = default;
  // A new advance call is about to issue its first operator.
  virtual void begin_call() {}
  // Enqueues operator `index` (0 .. total-1).  *launched = false when the operator had no device work.
  virtual int launch(int32_t index, bool* launched) = 0;
  // Places completion marker `slot` (0 .. kMarkRing-1) behind everything enqueued so far.
  virtual int mark(int slot) = 0;
  // Blocks the host until marker `slot` has completed on the device.
  virtual int wait_mark(int slot) = 0;
  // Blocks the host until everything enqueued has completed.
  virtual int drain() = 0;
  // True when the backend wants a marker behind every operator even without a launch-ahead bound
  // (per-operator timing).
  virtual bool wants_marks() const { return false; }
  // Operator number `issued` of this call has been enqueued (book-keeping hook).
  virtual void op_issued(int32_t /*issued*/, bool /*launched*/) {}
};

class TaskCore {
 public:
  TaskCore(int32_t total_ops, int32_t ops_per_layer, uint32_t boundary_mask)
      : total_(total_ops), per_layer_(ops_per_layer), mask_(boundary_mask) {}

  // Runs up to max_ops operators from the cursor.  kTaskOk: all issued and complete, more remain;
  // kTaskDone; kTaskPreempted: parked at an enabled boundary with the device drained; negative:
  // error, task idle again.  One thread at a time.
  int advance(OpBackend& be, int32_t max_ops, int32_t* ops_done) {
    if (ops_done) *ops_done = 0;
    {
      std::lock_guard<std::mutex> lk(mu_);
      if (state_ != TaskState::Idle) return kTaskErrState;
      state_ = TaskState::Running;
    }
    int32_t issued = 0;
    int32_t marked = 0;       // operators of this call with device work; the j-th one's marker is slot j % kMarkRing
    int result = kTaskOk;
    int32_t cur = cursor_.load(std::memory_order_relaxed);
    while (cur < total_ && issued < max_ops) {
      // Bound how far the host runs ahead of the device: at most launch_ahead operators with
      // device work are enqueued and not known complete (an operator without device work takes
      // no place in that window).  A slot is re-marked only after its previous marker was waited
      // for: launch_ahead <= kMarkRing.
      if (launch_ahead_ > 0 && marked >= launch_ahead_) {
        if (be.wait_mark((marked - launch_ahead_) % kMarkRing) != 0) { result = kTaskErrDevice; break; }
      }
      // Preemption check at the boundary behind the previous operator.
      const bool boundary = cur == 0 || ((mask_ >> ((cur - 1) % per_layer_)) & 1u);
      if (boundary && signal_.load(std::memory_order_acquire)) {
        if (be.drain() != 0) { result = kTaskErrDevice; break; }
        if (ops_done) *ops_done = issued;
        finish(TaskState::Parked, true);
        return kTaskPreempted;
      }
      if (issued == 0) be.begin_call();
      bool launched = true;
      if (be.launch(cur, &launched) != 0) { result = kTaskErrDevice; break; }
      // One marker per operator serves the launch-ahead bound (and the backend's timing); an
      // operator without device work places none and completes with its predecessor.
      if (launched && (launch_ahead_ > 0 || be.wants_marks())) {
        if (be.mark(marked % kMarkRing) != 0) { result = kTaskErrDevice; break; }
        ++marked;
      }
      be.op_issued(issued, launched);
      ++cur;
      cursor_.store(cur, std::memory_order_release);
      ++issued;
    }
    if (be.drain() != 0 && result >= 0) result = kTaskErrDevice;
    if (ops_done) *ops_done = issued;
    if (result < 0) {
      finish(TaskState::Idle, false);
      return result;
    }
    if (cur >= total_) {
      finish(TaskState::Done, true);
      return kTaskDone;
    }
    // A signal that arrived during the last operators of this call is honoured here: the device
    // is already quiescent.
    if (signal_.load(std::memory_order_acquire)) {
      finish(TaskState::Parked, true);
      return kTaskPreempted;
    }
    finish(TaskState::Idle, false);
    return kTaskOk;
  }

  // Raises the signal.  kTaskOk: the running advance will acknowledge; kTaskPreempted: the task
  // was idle and is parked now; kTaskDone; kTaskErrState: already parked.
  int preempt_signal() {
    std::lock_guard<std::mutex> lk(mu_);
    switch (state_) {
      case TaskState::Running: signal_.store(1, std::memory_order_release); return kTaskOk;
      case TaskState::Idle: state_ = TaskState::Parked; return kTaskPreempted;
      case TaskState::Done: return kTaskDone;
      case TaskState::Parked: return kTaskErrState;
    }
    return kTaskErrState;
  }

  // Blocks until the signal has been acknowledged (kTaskPreempted) or the task completed first
  // (kTaskDone).  kTaskErrState when the task is idle with nothing pending.
  int preempt_wait() {
    std::unique_lock<std::mutex> lk(mu_);
    for (;;) {
      if (state_ == TaskState::Parked) return kTaskPreempted;
      if (state_ == TaskState::Done) return kTaskDone;
      if (state_ == TaskState::Idle) {
        if (signal_.load(std::memory_order_acquire)) {   // the advance call ended between signal and wait
          signal_.store(0, std::memory_order_release);
          state_ = TaskState::Parked;
          return kTaskPreempted;
        }
        return kTaskErrState;
      }
      cv_.wait(lk);
    }
  }

  int resume() {
    std::lock_guard<std::mutex> lk(mu_);
    if (state_ != TaskState::Parked) return kTaskErrState;
    state_ = TaskState::Idle;
    return kTaskOk;
  }

  int set_launch_ahead(int32_t k) {
    if (k < 0 || k > kMarkRing) return kTaskErrInvalid;
    std::lock_guard<std::mutex> lk(mu_);
    if (state_ == TaskState::Running) return kTaskErrState;
    launch_ahead_ = k;
    return kTaskOk;
  }

  // Next operator to run.  May be read from any thread at any time.
  int32_t cursor() const { return cursor_.load(std::memory_order_acquire); }
  TaskState state() {
    std::lock_guard<std::mutex> lk(mu_);
    return state_;
  }
  // Runs fn() under the task's lock unless an advance call is in flight (then returns false).
  template <typename F> bool unless_running(F&& fn) {
    std::lock_guard<std::mutex> lk(mu_);
    if (state_ == TaskState::Running) return false;
    fn();
    return true;
  }
  int32_t total_ops() const { return total_; }

 private:
  void finish(TaskState st, bool ack) {
    std::lock_guard<std::mutex> lk(mu_);
    state_ = st;
    if (ack) signal_.store(0, std::memory_order_release);
    cv_.notify_all();
  }

  const int32_t total_, per_layer_;
  const uint32_t mask_;
  int32_t launch_ahead_ = 2;             // written only while no advance is in flight
  std::mutex mu_;
  std::condition_variable cv_;
  TaskState state_ = TaskState::Idle;    // guarded by mu_
  std::atomic<int> signal_{0};
  std::atomic<int32_t> cursor_{0};
};

}  // namespace fp
