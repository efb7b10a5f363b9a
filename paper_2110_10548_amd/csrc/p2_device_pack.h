// Packing of bandwidth-row entries: which local group (and its first device) touches a hardware
// unit, and how many groups of the whole system with that local id do.  Shared by the planner
// (host) and the cost code (device).
#pragma once
#include <cstdint>
#if defined(__HIPCC__)
#define P2_HD __host__ __device__
#else
#define P2_HD
#endif
namespace p2 {
P2_HD inline uint32_t entry_pack(uint32_t group, uint32_t base_dev, uint32_t cnt) { return (group << 19) | (base_dev << 10) | cnt; }
P2_HD inline uint32_t entry_cnt(uint32_t e) { return e & 0x3ffu; }
P2_HD inline uint32_t entry_base(uint32_t e) { return (e >> 10) & 0x1ffu; }
P2_HD inline uint32_t entry_group(uint32_t e) { return e >> 19; }
}  // namespace p2
