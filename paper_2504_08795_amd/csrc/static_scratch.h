// The library's static device scratch: see static_scratch.hip.
#pragma once
#include <cstddef>
#include <string>

// Size of the array, per GPU.  Holds the activation buffers and the split-K workspace of every configured network
// except VGG-16 (fp32: ResNet-50 9.6 MiB, MobileNetV2 8.2 MiB, ResNet-18 5 MiB).
#define DARIS_STATIC_SCRATCH_BYTES (16u << 20)

namespace daris {

// Looks up the device address of this GPU's copy of the array; `device` must be the current HIP device.  Once per
// device; later calls return at once.  Returns "" or an error text.
std::string static_scratch_init(int device);
// The address found by static_scratch_init for that device, or nullptr.
void* static_scratch_ptr(int device);

}  // namespace daris
