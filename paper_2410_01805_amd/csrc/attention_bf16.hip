// placeholder until the MFMA kernel lands
#include "kernels.h"
namespace locret {
void launch_attention_bf16(const Dims& D, const void* q, const void* Kx, const void* V, void* out, int T, int n_c,
                           float scale, hipStream_t st) {
  launch_attention_simple(D, q, Kx, V, out, T, n_c, scale, st);
}
}  // namespace locret
