// Shared between the code generator and the launcher: where each value sits in
// the kernel's argument block (an array of 8-byte slots passed by value).
#pragma once

#include <string>
#include <vector>

#include "ir.h"

namespace gr {

struct ArgLayout {
  std::vector<int> ptr;        // per access group: slot of the buffer pointer
  std::vector<int> base;       // per access group: slot of the base element offset
  std::vector<int> coef;       // per access group: first of `ncoef[g]` coefficient slots
  std::vector<int> ncoef;
  int out = 0;                 // output pointer
  int dims = 0;                // first of `rank` extents
  int consts = 0;              // first constant slot
  int extra = 0;               // kind-specific: GEMV {M, K, workspace, slabs}; REDUCE {outputs, length, workspace, splits};
                               // SCAN {lines, chunk length, workspace, chunks}
  int ocoef = 0;               // SCAN, MAP: first of `rank` output strides
  int obase = 0;               // MAP: element offset of the output's first element
  int total = 0;
};

ArgLayout arg_layout(const GroupPlan& g);

// 'Z': no leaf dimension follows this iteration dimension; '1': unit stride; 'G': anything else.
char access_class(const AccessGroup& ag, int dim);

// Whether loads of this access group carry the non-temporal hint.
bool nontemporal_group(const GroupPlan& g, int group);

}  // namespace gr
