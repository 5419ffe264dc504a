// Geometry shared by the kernels and by the host-side layout arithmetic (no HIP types here, so
// that the host logic also compiles with a plain C++ compiler).
//   group      = 4 consecutive coordinates (one 128-bit access, one Philox4x32 block)
//   tile       = 64 groups = 256 consecutive coordinates = what one wavefront handles at a time
//   superblock = 512 tiles; subset counts are scanned inside a superblock by one workgroup and
//                across superblocks by a second tiny kernel
//   line       = 128 bytes = 32 floats, the unit in which memory is written
//   block      = up to 8 replicas whose sparse values sit side by side in memory
#pragma once
#include <stdint.h>

namespace am {

constexpr uint32_t kTileCoords = 256;
constexpr uint32_t kTilesPerSuperblock = 512;
constexpr uint32_t kLineFloats = 32;
constexpr uint32_t kMaxReplicas = 32;
constexpr uint32_t kMaxBlockReplicas = 8;

}  // namespace am
