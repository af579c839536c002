// Host entry points of the full-Craftax variant, called by the C ABI in craftax.hip once the
// state's variant is known.  Every function returns 0 or a negative CRAFTAX_E_* code and, on
// error, a message in *err.  Nothing here synchronises except state_init.
#pragma once

#include <cstddef>
#include <cstdint>
#include <string>

#include "../../include/craftax.h"

namespace cf {
namespace host {

bool config_ok(const craftax_config* cfg, std::string* why);
size_t state_bytes(const craftax_config* cfg, int n);
size_t obs_bytes(const craftax_config* cfg);
int state_init(void* state, const craftax_config* cfg, int n, void* stream, std::string* err);
int reset(void* state, const craftax_config* cfg, int n, const uint64_t* seeds, void* stream, std::string* err);
// serve_slow: also launch the kernel that serves episodes which ended before their spare world existed
int step(void* state, const craftax_config* cfg, int n, const int32_t* actions, void* obs, float* reward, uint8_t* done,
         bool serve_slow, void* stream, std::string* err);
// checks a header read back from a blob against cfg and n: 0, or a CRAFTAX_E_* code and a message
int check_header(const void* header_bytes, const craftax_config* cfg, int n, std::string* err);
// where the metrics kernel finds achievements, t and episode (records as dwords) and the unlock counters
struct RecordLayout { const uint32_t* recs; int stride, ach, ach_words, t, episode; const uint32_t* unlocks; int unlock_stride; };
RecordLayout record_layout(const void* state, const craftax_config* cfg, int n);
// debug build: adds this translation unit's bounds record to report[4] and clears it
int debug_bounds(uint32_t report[4], std::string* err);
// LDS and thread needs of the kernels this configuration launches against the device's limits
int check_kernels(const craftax_config* cfg, std::string* err);
int rollout(void* state, const craftax_config* cfg, int n, const int32_t* actions, int steps, void* obs, float* reward, uint8_t* done,
            void* stream, std::string* err);
int observe(void* state, const craftax_config* cfg, int n, void* obs, void* stream, std::string* err);
int export_envs(const void* state, const craftax_config* cfg, int n, int first, int count, void* dumps, void* stream, std::string* err);
int import_envs(void* state, const craftax_config* cfg, int n, int first, int count, const void* dumps, void* stream, std::string* err);
int mutate_swap(void* state, const craftax_config* cfg, int n, int first, int count, uint64_t mutation_seed, uint32_t round,
                int restricted, int32_t* tries, void* stream, std::string* err);
int mutate_noise(void* state, const craftax_config* cfg, int n, int first, int count, uint16_t* theta, uint64_t mutation_seed, uint32_t round,
                 uint32_t amplitude, void* stream, std::string* err);

}  // namespace host
}  // namespace cf
