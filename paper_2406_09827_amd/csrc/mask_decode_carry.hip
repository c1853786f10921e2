// Decode mask estimation with the first or the last block of a branch as its representative:
// the variant that carries a node's score over to the child that shares its representative.
#include "mask_decode_impl.h"

namespace hipattn {

hipError_t launch_mask_decode_carry(const KParams &p, hipStream_t st) { return launch_mask_decode_variant<true>(p, st); }

}  // namespace hipattn
