// Process-wide tuning switches: a small table of named text values.  Each entry
// starts from the environment variable FUPR_<NAME IN CAPITALS>, read once when
// the table is first used, and changes afterwards only through fupr_tuning_set.
#include "tuning.h"

#include <cctype>
#include <cstdlib>
#include <cstring>
#include <mutex>

#include "fupr.h"

namespace fupr {
namespace {

constexpr size_t kValueBytes = 128;

struct Switch {
  const char* name;
  bool set;
  char value[kValueBytes];
};

Switch g_switches[] = {
    {"patch_tile", false, {0}},      // index of the 3 x 3 patch kernel's tile
    {"pipe_tile", false, {0}},       // index of the pipelined 1 x 1 kernel's tile
    {"pipe_order", false, {0}},      // that kernel's tiles: 0 a contiguous range per workgroup, 1 per XCD
    {"stream_tile", false, {0}},     // index of the streaming 1 x 1 kernel's tile
    {"stream_blocks", false, {0}},   // workgroups per compute unit that kernel is compiled for (1, 2)
    {"conv_tile", false, {0}},       // name of the general kernel's tile
    {"conv_patch", false, {0}},      // 0: 3 x 3 layers skip the patch kernel
    {"conv1x1_stream", false, {0}},  // 0: 1 x 1 layers skip the streaming kernel
    {"conv1x1_pipe", false, {0}},    // 0: 1 x 1 layers skip the pipelined kernel
    {"conv1x1_fuse", false, {0}},    // 0: no pairs of 1 x 1 convolutions in one launch
    {"pair_filters", false, {0}},    // most filters of such a pair's second convolution (up to 128)
    {"split", false, {0}},           // sub-batches of the per-operator schedule
    {"res_item", false, {0}},        // work-item shapes of the one-kernel schedule
    {"debug", false, {0}},           // non-empty: planner and HIP error text on stderr
};

std::mutex g_mutex;
std::once_flag g_env_once;

void read_environment() {
  for (Switch& s : g_switches) {
    char var[64] = "FUPR_";
    size_t n = std::strlen(var);
    for (const char* c = s.name; *c && n + 1 < sizeof(var); ++c) var[n++] = (char)std::toupper((unsigned char)*c);
    var[n] = 0;
    const char* e = std::getenv(var);
    if (e && *e && std::strlen(e) < kValueBytes) {
      std::strcpy(s.value, e);
      s.set = true;
    }
  }
}

Switch* find(const char* name) {
  std::call_once(g_env_once, read_environment);
  for (Switch& s : g_switches)
    if (std::strcmp(s.name, name) == 0) return &s;
  return nullptr;
}

}  // namespace

bool tuning_text(const char* name, char* out, size_t n) {
  Switch* s = find(name);
  if (!s || n == 0) return false;
  std::lock_guard<std::mutex> lock(g_mutex);
  if (!s->set) return false;
  std::strncpy(out, s->value, n - 1);
  out[n - 1] = 0;
  return true;
}

int tuning_int(const char* name, int unset) {
  char buf[kValueBytes];
  return tuning_text(name, buf, sizeof(buf)) ? std::atoi(buf) : unset;
}

bool tuning_off(const char* name) {
  char buf[kValueBytes];
  return tuning_text(name, buf, sizeof(buf)) && buf[0] == '0';
}

}  // namespace fupr

extern "C" fupr_status fupr_tuning_set(const char* name, const char* value) {
  if (!name) return FUPR_ERR_NULL;
  fupr::Switch* s = fupr::find(name);
  if (!s) return FUPR_ERR_ARG;
  if (value && std::strlen(value) >= fupr::kValueBytes) return FUPR_ERR_ARG;
  std::lock_guard<std::mutex> lock(fupr::g_mutex);
  s->set = value && *value;
  if (s->set) std::strcpy(s->value, value);
  return FUPR_OK;
}
