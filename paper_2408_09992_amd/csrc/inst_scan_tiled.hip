// Instantiates the batched catalogue-scan kernels (see the instance lists in kernels.hpp).
#define PQ_INSTANCE_TU
#include "kernels.hpp"
namespace pqk {
PQ_TILED_INSTANCES(PQ_TILED_DEFINE)
}
