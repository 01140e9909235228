// Plain types shared by the host scan (no HIP headers) and the kernel launchers.
#pragma once
#include <stdint.h>

namespace ivf {

// A host-side candidate (row already re-scored in fp64), handed to the merge kernel.
struct HostCand {
    double key;     // larger is nearer: inner product, or minus the squared distance
    int64_t id;
};

}  // namespace ivf
