#pragma once
#include <hip/hip_runtime.h>

namespace distdl {
// Brackets the kernel launches issued during its lifetime with two events on
// `st` when profiling is enabled (distdl_profile_enable).
class ProfScope {
 public:
  ProfScope(const char* name, hipStream_t st);
  ~ProfScope();
  ProfScope(const ProfScope&) = delete;
  ProfScope& operator=(const ProfScope&) = delete;

 private:
  hipStream_t st_;
  bool active_;
};
}  // namespace distdl
