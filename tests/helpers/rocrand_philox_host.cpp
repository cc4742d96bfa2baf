// Host-side call into rocRAND's public Philox4x32-10 engine (its state functions are
// __host__ __device__), used only as an independent library pin for the CPU oracle's Philox.
// Nothing here runs on a GPU.
#include <hip/hip_runtime.h>
#include <rocrand/rocrand_kernel.h>
#include <cstdint>

extern "C" void rocrand_philox_block(unsigned long long seed, unsigned long long subsequence,
                                     unsigned long long counter64, uint32_t out[4])
{
    rocrand_state_philox4x32_10 st;
    // offset counts 32-bit outputs; one counter increment yields four of them
    rocrand_init(seed, subsequence, 4ull * counter64, &st);
    uint4 v = rocrand4(&st);
    out[0] = v.x; out[1] = v.y; out[2] = v.z; out[3] = v.w;
}
