// Instantiates one group of short catalogue-scan kernels (see the instance lists in kernels.hpp).
#define PQ_INSTANCE_TU
#include "kernels.hpp"
namespace pqk {
PQ_SHORT_INSTANCES_C(PQ_SHORT_DEFINE)
}
