// Host-side registry of the kernel family: launch-function tables filled by the instance shards.
#pragma once
#include "ks_common.hpp"

namespace ks {

// variant index = akc*4 + bkc*2 + vec
typedef void (*LaunchFn)(const GemmParams &p, int grid, int variant, hipStream_t stream);

struct InstanceDesc {
    int id, core, bm, bn, bk, p1, p2, threads, splitK, ldsBytes, kw;
};

constexpr int kNumF32 = 64;
constexpr int kNumBf16 = 32;
constexpr int kShards = 16;

}  // namespace ks
