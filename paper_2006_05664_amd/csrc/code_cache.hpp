// Cache of compiled code objects, in memory and optionally in a directory: see code_cache.cpp.
#pragma once

#include <cstdint>
#include <string>
#include <vector>

namespace opevo {

// Everything a code object depends on, as one string: template name, hashes of the template
// texts, the fixed compiler options and the member's constants.
std::string code_cache_key(const std::string &tmpl, const std::string &defines);
bool code_cache_get(const std::string &key, std::vector<char> &code);
void code_cache_put(const std::string &key, const std::vector<char> &code);
int code_cache_configure(const char *dir, int64_t max_memory_bytes);
void code_cache_clear_memory();
void code_cache_stats(int64_t *hits, int64_t *disk_hits, int64_t *misses, int64_t *entries, int64_t *bytes);

}  // namespace opevo
