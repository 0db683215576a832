// Stand-in for the HIP runtime header when the scalar relaxation algebra (csrc/relax.h) is compiled for the host
// by tests/test_relax_host.py: the header needs nothing from HIP beyond the function qualifiers.
#pragma once
#include <math.h>
#define __device__
#define __forceinline__ inline
