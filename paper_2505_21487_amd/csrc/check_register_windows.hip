// Not part of the library: a translation unit that the build's code-generation
// check compiles to assembly (python -m paper_2505_21487_amd.build --check).
// It holds the main-kernel instantiations that keep their page-id windows in
// registers (page mode 3) and pins down which shapes those are.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <type_traits>

#include "../../include/gla_decode.h"
#include "common.hpp"
#include "tuned_device.hpp"
#include "tuned_main_kernel.hpp"

namespace gla {

// Every (d_v, NG, WPG, KS) the host dispatches has room for LDS windows, except
// the 512-dim latent with two row slabs per workgroup: that one runs page mode 3.
static_assert(tuned_windows_fit(512, 1, 1, 2) && !tuned_windows_fit(512, 1, 2, 2), "512-dim latent");
static_assert(tuned_windows_fit(256, 1, 1, 1) && tuned_windows_fit(256, 1, 2, 1) && tuned_windows_fit(256, 1, 4, 1) &&
                  tuned_windows_fit(256, 2, 1, 1) && tuned_windows_fit(256, 2, 2, 1),
              "256-dim latent heads");
static_assert(tuned_windows_fit(128, 1, 1, 1) && tuned_windows_fit(128, 1, 2, 1) && tuned_windows_fit(128, 1, 4, 1) &&
                  tuned_windows_fit(128, 2, 1, 1) && tuned_windows_fit(128, 2, 2, 1) && tuned_windows_fit(128, 4, 1, 1),
              "128-dim tied heads");

template __global__ void tuned_main_kernel<512, 512, 64, 1, 2, 2, kTok, tuned_stages(512, 1, 2, 2), 3, true>(DevParams);
template __global__ void tuned_main_kernel<512, 512, 64, 1, 2, 2, kTok, tuned_stages(512, 1, 2, 2), 3, false>(DevParams);

}  // namespace gla
