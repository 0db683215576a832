// Host harness around the library's scalar relaxation algebra (csrc/relax.h), driven by tests/test_relax_host.py:
// reads "op l u" lines, prints the two lines (kL cL kU cU) the device code would use (leaky: slope 0.1 on x < 0).
#include <stdio.h>
#include <string.h>
#include "relax.h"

int main() {
  char op[16];
  double l, u;
  while (scanf("%15s %lf %lf", op, &l, &u) == 3) {
    tv::Line2 r;
    if (!strcmp(op, "relu")) r = tv::relax_relu(l, u);
    else if (!strcmp(op, "tanh")) r = tv::relax_tanh(l, u);
    else if (!strcmp(op, "exp")) r = tv::relax_exp(l, u);
    else if (!strcmp(op, "recip")) r = tv::relax_recip(l, u);
    else if (!strcmp(op, "sqrt")) r = tv::relax_sqrt(l, u);
    else if (!strcmp(op, "square")) r = tv::relax_square(l, u);
    else if (!strcmp(op, "leaky")) r = tv::relax_leaky_relu(l, u, 0.1);
    else if (!strcmp(op, "silu")) {
      // the chain's form in x, printed as the two lines it gives for a neuron whose own lines coincide
      const tv::Form f = tv::silu_form(l, u);
      r = tv::Line2{f.pL + f.qL, f.cL, f.pU + f.qU, f.cU};
    }
    else return 2;
    printf("%.17g %.17g %.17g %.17g\n", r.kL, r.cL, r.kU, r.cU);
  }
  return 0;
}
