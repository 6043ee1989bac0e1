// The attention layer's context, shared by its forward (moa.hip) and backward (moa_bwd.hip) entry points.
#pragma once

#include "common.h"

struct dsmoe_moa_ctx {
  dsmoe_moa_desc desc;
  dsmoe_ctx inner;          // descriptor and CU count for the shared launchers; owns nothing
  char* workspace;
  size_t workspace_bytes;
  // workspace offsets: scores [T, E] f32, masks, selected counts, Q [E][T][hd], weighted outputs Cs [T][E hd];
  // for the backward pass also the unweighted outputs C [T][E hd] and lse [E][n_head][T] f32
  size_t o_probs, o_mask, o_cnt, o_q, o_cs, o_c, o_lse, total;
  // shape of the last forward call with every expert active (-1: none); the backward pass needs exactly that one
  int32_t saved_T, saved_L;
  float saved_scale;
  char err[256];
};
