#include "fiber.h"

#include <sys/mman.h>
#include <unistd.h>

#include <cstdint>
#include <cstring>
#include <exception>
#include <vector>

#if !defined(__x86_64__) && !defined(__HIP_DEVICE_COMPILE__)
#error "the fiber context switch is written for x86-64 (System V calling convention)"
#endif

// acrobat_fiber_switch(void** save_sp, void* load_sp): pushes the callee-saved registers, stores
// the stack pointer to *save_sp, loads load_sp, pops the callee-saved registers of the context
// that was suspended there and returns into it.  No system call (the signal mask is not touched),
// about 20 ns per switch.
#if !defined(__HIP_DEVICE_COMPILE__)
asm(R"(
.text
.globl acrobat_fiber_switch
.hidden acrobat_fiber_switch
.type acrobat_fiber_switch,@function
acrobat_fiber_switch:
    pushq %rbp
    pushq %rbx
    pushq %r12
    pushq %r13
    pushq %r14
    pushq %r15
    movq %rsp, (%rdi)
    movq %rsi, %rsp
    popq %r15
    popq %r14
    popq %r13
    popq %r12
    popq %rbx
    popq %rbp
    ret
.size acrobat_fiber_switch,.-acrobat_fiber_switch
)");
#endif
extern "C" void acrobat_fiber_switch(void** save_sp, void* load_sp);

namespace acrobat {

namespace {
thread_local FiberScheduler* tl_scheduler = nullptr;  // the scheduler whose run() is active on this thread

// Stacks outlive their scheduler: mapping one costs two system calls and its first use a page
// fault, more than everything else a short-lived fiber does.  Per thread, all of one size.
constexpr size_t kPooledStacks = 65536;  // (address space and the pages a fiber touched: a few KB each)
struct StackPool {
  size_t bytes = 0;  // mapping size of the pooled stacks
  std::vector<char*> free;
  ~StackPool() {
    for (char* m : free) munmap(m, bytes);
  }
};
thread_local StackPool tl_stacks;
}

FiberScheduler::FiberScheduler(size_t stack_bytes) {
  const size_t page = (size_t)sysconf(_SC_PAGESIZE);
  stack_bytes_ = (stack_bytes + page - 1) / page * page;
}

FiberScheduler::~FiberScheduler() {
  const size_t page = (size_t)sysconf(_SC_PAGESIZE);
  const size_t bytes = stack_bytes_ + page;
  if (tl_stacks.bytes != bytes) {
    for (char* m : tl_stacks.free) munmap(m, tl_stacks.bytes);
    tl_stacks.free.clear();
    tl_stacks.bytes = bytes;
  }
  for (Fiber* f : all_) {
    if (f->stack) {
      if (tl_stacks.free.size() < kPooledStacks) tl_stacks.free.push_back(f->stack);
      else munmap(f->stack, bytes);
    }
    delete f;
  }
}

FiberScheduler::Fiber* FiberScheduler::acquire() {
  if (!idle_.empty()) {
    Fiber* f = idle_.back();
    idle_.pop_back();
    return f;
  }
  const size_t page = (size_t)sysconf(_SC_PAGESIZE);
  if (tl_stacks.bytes == stack_bytes_ + page && !tl_stacks.free.empty()) {
    Fiber* f = new Fiber();
    f->stack = tl_stacks.free.back();
    tl_stacks.free.pop_back();
    all_.push_back(f);
    return f;
  }
  // untouched pages cost nothing; the lowest page is a guard: running off the stack faults at once
  void* m = mmap(nullptr, stack_bytes_ + page, PROT_READ | PROT_WRITE, MAP_PRIVATE | MAP_ANONYMOUS | MAP_NORESERVE | MAP_STACK, -1, 0);
  if (m == MAP_FAILED) return nullptr;
  (void)mprotect(m, page, PROT_NONE);
  Fiber* f = new Fiber();
  f->stack = static_cast<char*>(m);
  all_.push_back(f);
  return f;
}

void FiberScheduler::retire(Fiber* f) {
  if (f->fn) f->fn = nullptr;
  idle_.push_back(f);
}

// First frame of every fiber.  Never returns: when fn is done the fiber switches away for good.
void FiberScheduler::entry() {
  FiberScheduler* s = tl_scheduler;
  Fiber* f = s->current_;
  try {
    if (f->plain) f->plain(f->arg);
    else f->fn();
  } catch (const std::exception& e) {
    if (s->error_.empty()) s->error_ = e.what();
  } catch (...) {
    if (s->error_.empty()) s->error_ = "unknown exception in a fiber";
  }
  f->done = true;
  acrobat_fiber_switch(&f->sp, s->main_sp_);
  __builtin_trap();  // a finished fiber is never resumed
}

void FiberScheduler::make_runnable(Fiber* f) {
  f->done = false;
  // initial frame: six zeroed callee-saved registers, then the address the first switch returns
  // to; the stack pointer is then 8 modulo 16, as right after a call instruction
  const size_t page = (size_t)sysconf(_SC_PAGESIZE);
  uintptr_t top = reinterpret_cast<uintptr_t>(f->stack + page + stack_bytes_) & ~(uintptr_t)15;
  uint64_t* sp = reinterpret_cast<uint64_t*>(top);
  *--sp = 0;                                             // where entry's caller would be
  *--sp = reinterpret_cast<uint64_t>(&FiberScheduler::entry);
  for (int i = 0; i < 6; ++i) *--sp = 0;
  f->sp = sp;
  runnable_.push_back(f);
  ++n_spawned_;
}

bool FiberScheduler::spawn(std::function<void()> fn) {
  Fiber* f = acquire();
  if (!f) return false;
  f->fn = std::move(fn);
  f->plain = nullptr;
  make_runnable(f);
  return true;
}

bool FiberScheduler::spawn(void (*fn)(void*), const void* arg, size_t arg_bytes) {
  if (arg_bytes > kInlineArg) return false;
  Fiber* f = acquire();
  if (!f) return false;
  f->plain = fn;
  std::memcpy(f->arg, arg, arg_bytes);
  make_runnable(f);
  return true;
}

void FiberScheduler::block() {
  Fiber* f = current_;
  if (!f) return;
  acrobat_fiber_switch(&f->sp, main_sp_);
}

void FiberScheduler::run() {
  FiberScheduler* outer = tl_scheduler;
  tl_scheduler = this;
  while (!runnable_.empty()) {
    Fiber* f = runnable_.front();
    runnable_.pop_front();
    // with thousands of fibers each one's frames have left the cache by the time its turn comes:
    // fetch those of a fiber a few turns ahead
    constexpr size_t kAhead = 4;  // (a fiber's turn is shorter than a memory access)
    if (runnable_.size() >= kAhead) {
      const char* next = static_cast<const char*>(runnable_[kAhead - 1]->sp);
      __builtin_prefetch(next);
      __builtin_prefetch(next + 64);
      __builtin_prefetch(next + 128);
      __builtin_prefetch(next + 192);
    }
    current_ = f;
    ++n_switches_;
    acrobat_fiber_switch(&main_sp_, f->sp);
    current_ = nullptr;
    if (f->done) retire(f);
    else blocked_.push_back(f);
  }
  tl_scheduler = outer;
}

void FiberScheduler::release() {
  for (Fiber* f : blocked_) runnable_.push_back(f);
  blocked_.clear();
}

}  // namespace acrobat
