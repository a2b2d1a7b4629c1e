// Network geometry (Section 3 layer list) and the internal parameter layout.
//
// Activations are channel-last (NHWC) so that the reduction index of every
// implicit GEMM runs over contiguous memory; weights are kept in the matching
// order:
//   conv1.W [32][c=4][p=8][q=8]      (input is the uint8 CHW frame stack)
//   conv2.W [64][p=4][q=4][c=32]
//   conv3.W [64][p=3][q=3][c=64]
//   fc1.W   [512][(h*7+w)*64 + c]
//   head    as in the canonical blob
// Tensor offsets inside the blob are the canonical ones; only the order inside
// conv2.W, conv3.W and fc1.W differs.
#pragma once
#include <stdint.h>

namespace net {
constexpr int FRAME = 84 * 84;          // bytes per frame
constexpr int STATE = 4 * FRAME;        // bytes per stacked state
constexpr int A1 = 20 * 20 * 32;        // conv1 output per sample
constexpr int A2 = 9 * 9 * 64;          // conv2 output per sample
constexpr int A3 = 7 * 7 * 64;          // conv3 output per sample (= fc1 input)
constexpr int HID = 512;

constexpr int64_t C1W = 0, C1B = 8192;
constexpr int64_t C2W = 8224, C2B = 40992;
constexpr int64_t C3W = 41056, C3B = 77920;
constexpr int64_t F1W = 77984, F1B = 1683616;
constexpr int64_t HEAD = 1684128;

constexpr int64_t L1N = 8224;           // conv1 W+b
constexpr int64_t L2N = 32832;          // conv2 W+b
constexpr int64_t L3N = 36928;          // conv3 W+b
constexpr int64_t L4N = 1606144;        // fc1 W+b

inline int64_t head_count(int K, int dueling) { return (int64_t)(K + (dueling ? 1 : 0)) * (HID + 1); }
inline int64_t param_count(int K, int dueling) { return HEAD + head_count(K, dueling); }

#ifdef __HIPCC__
// Workgroups are handed to the eight accelerator dies of the package round-robin in dispatch
// order (x fastest, then y, then z), and each die has an L2 of its own.  tile_of_workgroup turns
// the dispatch-order number of this workgroup into a tile number such that every die works on
// one contiguous range of tile numbers; the kernels number tiles that share operands next to
// each other, so they meet in one L2 instead of fetching the operand once per die.  The map
// is a bijection on [0, total) whatever the hardware does, so it can only change locality.
__device__ __forceinline__ int tile_of_workgroup()
{
    const int total = gridDim.x * gridDim.y * gridDim.z;
    const int id = blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z);
    const int die = id & 7, slot = id >> 3;
    const int q = total >> 3, r = total & 7;  // die d receives q + (d < r) workgroups
    return die * q + (die < r ? die : r) + slot;
}
#endif
}  // namespace net
