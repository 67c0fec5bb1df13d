// Host-side probe of AMD's open-source rocRAND Philox4x32-10 engine (its
// public device API is also callable on the host).  Used only by the oracle's
// pin tests as an independent opinion on the generator.  Built with g++:
//   g++ -O1 -shared -fPIC -D__HIP_PLATFORM_AMD__ -I/opt/rocm/include
#include <hip/hip_runtime.h>
#include <rocrand/rocrand_philox4x32_10.h>
#include <cstdint>

extern "C" void rocrand_philox_next4(uint64_t seed, uint64_t subsequence, uint64_t offset,
                                     uint32_t out[4]) {
    rocrand_device::philox4x32_10_engine engine(seed, subsequence, offset);
    const uint4 o = engine.next4();
    out[0] = o.x; out[1] = o.y; out[2] = o.z; out[3] = o.w;
}
