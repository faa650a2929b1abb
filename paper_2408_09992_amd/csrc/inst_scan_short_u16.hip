// Instantiates the short catalogue-scan kernels for two-byte sub-ids (see the instance lists in kernels.hpp).
#define PQ_INSTANCE_TU
#include "kernels.hpp"
namespace pqk {
PQ_SHORT16_INSTANCES(PQ_SHORT16_DEFINE)
}
