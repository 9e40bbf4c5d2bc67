// Winner cache shared by the kernels of this library (internal; nothing here crosses the C ABI).
// The cache file holds one line per (environment, shape bucket): the name of the fastest compiled
// instance and its time (the paper's requirement list: tuning results are kept in a reusable cache
// that records the environment they were measured in).  Attention buckets resolve their winner to an
// instance id when the file is loaded; every other kernel kind looks its winner up by name.
#pragma once
#include <string>

namespace attn {

std::string environment_key();
// Replaces or adds the line of (this environment, key) in the file at `path` (atomic replace).
// Returns an attn_status.
int merge_cache_line(const char *path, const std::string &key, const std::string &instance_name, double us);
// Winners of kernel kinds other than attention, by bucket key.
void store_named_winner(const std::string &key, const std::string &instance_name);
bool lookup_named_winner(const std::string &key, std::string *instance_name);
// Reads $ATTN_TUNE_CACHE once per process (no-op afterwards).
void load_env_cache_once();

}  // namespace attn
