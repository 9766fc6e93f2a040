// Backward of Attn-QAT (Alg. 3) -- placeholder translation unit, filled in next.
#include "common.hpp"
#include "kernels.hpp"
namespace aq {
int launch_delta(const void*, const float*, int, int, int, float*, hipStream_t) { return -1; }
int launch_bwd_dq(const void*, const void*, const void*, const void*, const void*, const float*, const float*,
                  int, int, int, int, int, bool, void*, hipStream_t) { return -1; }
int launch_bwd_dkdv(const void*, const void*, const void*, const void*, const void*, const void*, const float*,
                    const float*, int, int, int, int, int, bool, void*, void*, hipStream_t) { return -1; }
}
