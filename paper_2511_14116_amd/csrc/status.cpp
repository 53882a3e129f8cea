// Status messages, option table and version of the C ABI.
#include <cstdio>
#include <cstring>

#include "fs_internal.h"

namespace fs {

static thread_local char g_msg[512] = "";

fs_status fail(fs_status st, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_msg, sizeof(g_msg), fmt, ap);
  va_end(ap);
  return st;
}

Options& options() {
  static Options o{4, 2, 1, 8};
  return o;
}

}  // namespace fs

extern "C" const char* fs_last_error(void) { return fs::g_msg; }

extern "C" int32_t fs_abi_version(void) { return FS_ABI_VERSION; }

extern "C" fs_status fs_set_option(const char* key, int32_t value) {
  if (!key) return fs::fail(FS_EINVAL, "fs_set_option: key is NULL");
  if (!strcmp(key, "waves_per_group")) {
    if (value != 1 && value != 2 && value != 4)
      return fs::fail(FS_EINVAL, "waves_per_group must be 1, 2 or 4 (got %d)", value);
    fs::options().waves_per_group = value;
    return FS_OK;
  }
  if (!strcmp(key, "prefetch_pages")) {
    if (value < 1 || value > 3)
      return fs::fail(FS_EINVAL, "prefetch_pages must be in [1, 3] (got %d)", value);
    fs::options().prefetch_pages = value;
    return FS_OK;
  }
  if (!strcmp(key, "prefill_col_tiles")) {
    if (value != 1 && value != 2 && value != 4)
      return fs::fail(FS_EINVAL, "prefill_col_tiles must be 1, 2 or 4 (got %d)", value);
    fs::options().prefill_col_tiles = value;
    return FS_OK;
  }
  if (!strcmp(key, "prefill_waves")) {
    if (value != 4 && value != 8)
      return fs::fail(FS_EINVAL, "prefill_waves must be 4 or 8 (got %d)", value);
    fs::options().prefill_waves = value;
    return FS_OK;
  }
  return fs::fail(FS_EINVAL, "fs_set_option: unknown key '%s'", key);
}

extern "C" int32_t fs_get_option(const char* key) {
  if (!key) return -1;
  if (!strcmp(key, "waves_per_group")) return fs::options().waves_per_group;
  if (!strcmp(key, "prefetch_pages")) return fs::options().prefetch_pages;
  if (!strcmp(key, "prefill_col_tiles")) return fs::options().prefill_col_tiles;
  if (!strcmp(key, "prefill_waves")) return fs::options().prefill_waves;
  return -1;
}
