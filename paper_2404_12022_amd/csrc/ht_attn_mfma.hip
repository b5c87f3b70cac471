// Tree-masked attention on CDNA4 matrix cores (bf16).  Placeholder: not yet enabled.
#include "ht_common.h"

namespace ht {

bool attn_mfma_supported(int M, int Hq, int Hkv, int hd) {
  (void)M; (void)Hq; (void)Hkv; (void)hd;
  return false;
}
size_t attn_mfma_scratch_bytes(int M, int Hq, int hd) {
  (void)M; (void)Hq; (void)hd;
  return 256;
}
hipError_t launch_attn_mfma(const void*, const void*, const void*, int, int, int, TreeDev, int, int, int, void*, void*,
                            hipStream_t) {
  return hipErrorNotSupported;
}

}  // namespace ht
