// Cooperative fibers on the calling thread (section 4.2).
//
// A program with tensor-dependent control flow cannot be run to its end before anything is
// evaluated: it stops wherever it needs the value of a tensor.  Run one instance after the other,
// every such stop would trigger an evaluation holding one operator.  So every instance - and,
// fork-join style, every part of an instance that may proceed on its own, such as the subtrees of a
// recursion - runs on a fiber: an execution stack of its own, switched by hand.  All fibers advance
// until each has finished or waits for a value; then the graph built so far is evaluated in
// batches, the waiting fibers become runnable again, and so on.
//
// Single threaded: everything here is called from one thread; spawn() and block() may be called
// from inside a fiber, run() and release() only from outside.
#pragma once
#include <cstddef>
#include <deque>
#include <functional>
#include <string>
#include <vector>

namespace acrobat {

class FiberScheduler {
 public:
  explicit FiberScheduler(size_t stack_bytes = 64 << 10);
  ~FiberScheduler();
  FiberScheduler(const FiberScheduler&) = delete;
  FiberScheduler& operator=(const FiberScheduler&) = delete;

  // A new runnable fiber that will call fn.  False if no stack could be allocated.
  bool spawn(std::function<void()> fn);
  // The same for a plain function and up to kInlineArg bytes of argument, copied into the fiber (no
  // allocation: forking is the most frequent operation of a recursive program).
  static constexpr size_t kInlineArg = 48;
  bool spawn(void (*fn)(void*), const void* arg, size_t arg_bytes);
  // Inside a fiber: suspend until the next release().
  void block();
  // Runs the runnable fibers, first come first served, including those spawned meanwhile, until
  // every fiber has finished or blocked.
  void run();
  // Fibers waiting in block().
  size_t blocked() const { return blocked_.size(); }
  // Every blocked fiber becomes runnable, in the order in which they blocked.
  void release();
  bool in_fiber() const { return current_ != nullptr; }
  // Text of the first exception that reached the top of a fiber (empty: none).
  const std::string& error() const { return error_; }
  size_t spawned() const { return n_spawned_; }
  size_t switches() const { return n_switches_; }

 private:
  struct Fiber {
    void* sp = nullptr;      // saved stack pointer while suspended
    char* stack = nullptr;   // mapping: guard page + stack_bytes_
    std::function<void()> fn;
    void (*plain)(void*) = nullptr;
    alignas(16) unsigned char arg[kInlineArg];
    bool done = false;
  };
  static void entry();
  Fiber* acquire();
  void retire(Fiber* f);
  void make_runnable(Fiber* f);

  size_t stack_bytes_;
  void* main_sp_ = nullptr;
  Fiber* current_ = nullptr;
  std::deque<Fiber*> runnable_;
  std::vector<Fiber*> blocked_;
  std::vector<Fiber*> idle_;  // finished fibers whose stacks are reused
  std::vector<Fiber*> all_;
  std::string error_;
  size_t n_spawned_ = 0, n_switches_ = 0;
};

}  // namespace acrobat
