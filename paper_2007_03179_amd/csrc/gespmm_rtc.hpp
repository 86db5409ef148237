// User-defined reduce operations compiled at run time (the paper's general operation, Eq. 1 and
// Section IV-A: the user's initialisation and reduce functions are inlined into the kernel when it
// is compiled; here that compilation happens inside the running process, with hiprtc).
//
// The user's source text defines a struct with identity(), step(acc, a, b) and merge(x, y), exactly
// as for include/gespmm_custom.hpp.  It is compiled together with the text of gespmm_device.hpp
// (embedded in this library when it is built) and the chunk kernel is instantiated for the
// CustomRows policy of that struct, once per launch shape that is actually used, on first use.
// hiprtc itself is loaded on first use: the rest of the library does not depend on it.
#pragma once

#include <dlfcn.h>
#include <hip/hiprtc.h>

#include <map>
#include <mutex>
#include <string>
#include <tuple>
#include <vector>

#include "gespmm_kernels.hpp"

namespace gespmm_detail {

static const char kDeviceHeaderText[] =
#include "gespmm_device_source.inc"
    ;

// The entry points of libhiprtc this file uses, resolved once.
struct HiprtcApi {
  decltype(&hiprtcCreateProgram) create = nullptr;
  decltype(&hiprtcDestroyProgram) destroy = nullptr;
  decltype(&hiprtcAddNameExpression) add_name = nullptr;
  decltype(&hiprtcCompileProgram) compile = nullptr;
  decltype(&hiprtcGetProgramLogSize) log_size = nullptr;
  decltype(&hiprtcGetProgramLog) log = nullptr;
  decltype(&hiprtcGetLoweredName) lowered_name = nullptr;
  decltype(&hiprtcGetCodeSize) code_size = nullptr;
  decltype(&hiprtcGetCode) code = nullptr;
  bool ok = false;
};

inline const HiprtcApi& hiprtc_api() {
  static const HiprtcApi api = [] {
    HiprtcApi a;
    void* lib = dlopen("libhiprtc.so", RTLD_NOW | RTLD_LOCAL);
    if (!lib) lib = dlopen("/opt/rocm/lib/libhiprtc.so", RTLD_NOW | RTLD_LOCAL);
    if (!lib) return a;
#define GESPMM_RESOLVE(field, symbol) a.field = reinterpret_cast<decltype(a.field)>(dlsym(lib, #symbol));
    GESPMM_RESOLVE(create, hiprtcCreateProgram)
    GESPMM_RESOLVE(destroy, hiprtcDestroyProgram)
    GESPMM_RESOLVE(add_name, hiprtcAddNameExpression)
    GESPMM_RESOLVE(compile, hiprtcCompileProgram)
    GESPMM_RESOLVE(log_size, hiprtcGetProgramLogSize)
    GESPMM_RESOLVE(log, hiprtcGetProgramLog)
    GESPMM_RESOLVE(lowered_name, hiprtcGetLoweredName)
    GESPMM_RESOLVE(code_size, hiprtcGetCodeSize)
    GESPMM_RESOLVE(code, hiprtcGetCode)
#undef GESPMM_RESOLVE
    a.ok = a.create && a.destroy && a.add_name && a.compile && a.log_size && a.log && a.lowered_name && a.code_size && a.code;
    return a;
  }();
  return api;
}

// Compiles `source` (which may include "gespmm_device.hpp") for the architecture `arch`.  name_expression: a
// template instantiation to emit and look up, or empty; plain_name: an extern "C" kernel to look up
// instead.  On success *code holds the code object and *symbol the name to ask the module for.
inline int rtc_compile(const std::string& source, const std::string& arch, const std::string& name_expression,
                       const std::string& plain_name, std::vector<char>* code, std::string* symbol, std::string* log) {
  const HiprtcApi& rtc = hiprtc_api();
  if (!rtc.ok) {
    if (log) *log = "libhiprtc.so could not be loaded";
    return GESPMM_ERR_NO_RTC;
  }
  const char* header_names[] = {"gespmm_device.hpp"};
  const char* header_texts[] = {kDeviceHeaderText};
  hiprtcProgram program = nullptr;
  if (rtc.create(&program, source.c_str(), "gespmm_user_reduce.hip", 1, header_texts, header_names) != HIPRTC_SUCCESS)
    return GESPMM_ERR_COMPILE;
  int status = GESPMM_OK;
  if (!name_expression.empty() && rtc.add_name(program, name_expression.c_str()) != HIPRTC_SUCCESS) status = GESPMM_ERR_COMPILE;
  if (status == GESPMM_OK) {
    const std::string arch_option = "--offload-arch=" + arch;
    // the same code generation options as the build of the library itself
    const char* options[] = {arch_option.c_str(), "-O3", "-std=c++17", "-munsafe-fp-atomics",
                             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"};
    const hiprtcResult compiled = rtc.compile(program, (int)(sizeof(options) / sizeof(options[0])), options);
    size_t log_bytes = 0;
    if (log && rtc.log_size(program, &log_bytes) == HIPRTC_SUCCESS && log_bytes > 1) {
      log->assign(log_bytes, '\0');
      rtc.log(program, &(*log)[0]);
    }
    if (compiled != HIPRTC_SUCCESS) status = GESPMM_ERR_COMPILE;
  }
  if (status == GESPMM_OK) {
    if (!name_expression.empty()) {
      const char* lowered = nullptr;
      if (rtc.lowered_name(program, name_expression.c_str(), &lowered) != HIPRTC_SUCCESS || !lowered) status = GESPMM_ERR_COMPILE;
      else *symbol = lowered;
    } else {
      *symbol = plain_name;
    }
  }
  if (status == GESPMM_OK) {
    size_t bytes = 0;
    if (rtc.code_size(program, &bytes) != HIPRTC_SUCCESS || bytes == 0) status = GESPMM_ERR_COMPILE;
    else {
      code->assign(bytes, '\0');
      if (rtc.code(program, code->data()) != HIPRTC_SUCCESS) status = GESPMM_ERR_COMPILE;
    }
  }
  rtc.destroy(&program);
  return status;
}

inline bool is_identifier(const char* name) {
  if (!name || !*name) return false;
  for (const char* c = name; *c; ++c) {
    const bool letter = (*c >= 'a' && *c <= 'z') || (*c >= 'A' && *c <= 'Z') || *c == '_';
    const bool digit = *c >= '0' && *c <= '9';
    if (!(letter || (digit && c != name) || (*c == ':' && c != name))) return false;   // Name or ns::Name
  }
  return true;
}

}  // namespace gespmm_detail

// One user-defined reduce operation: its source, its identity value, and the kernels built so far.
struct gespmm_custom_op {
  std::string source;       // "#include gespmm_device.hpp" + the user's text
  std::string name;         // the user's struct
  std::string arch;         // architecture of the device the operation was created on
  int device = 0;
  float identity = 0.0f;
  struct Built {
    hipModule_t module = nullptr;
    hipFunction_t function = nullptr;
  };
  std::mutex lock;          // guards `kernels`
  std::map<std::tuple<int, int, int, int>, Built> kernels;   // (vec, G, T, whole-row path) -> loaded kernel

  // The chunk kernel for CustomRows<name, vec, T> with slots of G lanes; compiled and loaded on first use.
  int kernel_for(int vec, int G, int T, bool whole_rows, hipFunction_t* out, std::string* log) {
    std::lock_guard<std::mutex> guard(lock);
    const auto key = std::make_tuple(vec, G, T, whole_rows ? 1 : 0);
    auto found = kernels.find(key);
    if (found == kernels.end()) {
      const std::string expression = "gespmm_detail::chunk_kernel<gespmm_detail::CustomRows<" + name + ", " + std::to_string(vec) +
                                     ", " + std::to_string(T) + ">, " + std::to_string(vec) + ", " + std::to_string(G) + ", " +
                                     std::to_string(T) + ", false, " + (whole_rows ? "true" : "false") + ">";
      std::vector<char> code;
      std::string symbol;
      const int compiled = gespmm_detail::rtc_compile(source, arch, expression, "", &code, &symbol, log);
      if (compiled != GESPMM_OK) return compiled;
      Built built;
      if (hipModuleLoadData(&built.module, code.data()) != hipSuccess) return GESPMM_ERR_HIP;
      if (hipModuleGetFunction(&built.function, built.module, symbol.c_str()) != hipSuccess) {
        (void)hipModuleUnload(built.module);
        return GESPMM_ERR_HIP;
      }
      found = kernels.emplace(key, built).first;
    }
    *out = found->second.function;
    return GESPMM_OK;
  }
};

namespace gespmm_detail {

inline int rtc_launch(void* context, const gespmm_plan_t& plan, const KernelArgs& args, hipStream_t stream) {
  gespmm_custom_op* op = static_cast<gespmm_custom_op*>(context);
  hipFunction_t function = nullptr;
  const int built = op->kernel_for(plan.vec, plan.lanes_per_row, plan.tiles_per_lane, plan.row_window > 0, &function, nullptr);
  if (built != GESPMM_OK) return built;
  KernelArgs copy = args;
  void* params[] = {&copy};
  if (hipModuleLaunchKernel(function, (unsigned)plan.grid_x, (unsigned)plan.col_blocks, 1, kBlock, 1, 1, (unsigned)plan.lds_bytes,
                            stream, params, nullptr) != hipSuccess)
    return GESPMM_ERR_HIP;
  return GESPMM_OK;
}

}  // namespace gespmm_detail
