// kernels.hpp -- HIP kernels of the STAND speculation step for gfx950 (wave64), one header per part:
//
//   wave_ops.hpp     limits, layouts, wave-level reductions, the accept / reject sequence of a node
//   row_pass.hpp     row_pass_kernel     softmax statistics + top-K of every logits row in one streaming
//                                        pass, and the accept/reject outcome of the row's tree node
//                                                                              (paper Sec. 4.1, 3.2)
//   path_pass.hpp    path_exact_kernel   exact integer partial sums of the rows on the accepted path;
//                                        walks the path and gathers the stop node's proposal (Sec. 3.2)
//                    path_finish_kernel  observation of each path row with the exact normaliser, replay
//                                        of the stop node, resampled token by inverting the residual's
//                                        cumulative integer mass; claims the table slots of the merge
//                                                                              (paper Sec. 3.2, 4.1)
//                    commit_scan_kernel  top-K of caller-given rows (update without verify)
//   table_merge.hpp  merge_apply_kernel  running-mean merge into the open-addressing table (Sec. 4.1)
//   draft.hpp        draft_kernel        multi-level lookup + Gumbel-Top-K along the static tree (Sec. 4.2)
//   step_fused.hpp   stand_step_kernel   the whole step in one launch: rows of the tree's upper levels, then
//                                        the dependent tail beside the remaining rows (bounded waits on
//                                        device-scope counters)
//   aux_kernels.hpp  fills, copies, tree packing, table export
//
// The row pass is the only kernel that touches all of the logits; it is bound by HBM bandwidth.
// Its softmax normaliser uses the hardware exp2 and float accumulation (relative error below
// the 5e-5 bound assumed here); every accept test whose margin is inside that bound, and
// every probability that is stored in the table or used for resampling, is recomputed with
// the exact integer normaliser of numeric.hpp, so all decisions are those of exact arithmetic.
// The kernels after the row pass are chains of dependent memory round trips over little data;
// their workgroups exchange data only across kernel boundaries.  stand_step_kernel runs the same
// device functions in one launch and orders them with counters instead.
#pragma once
#include "numeric.hpp"
#include "wave_ops.hpp"
#include "row_pass.hpp"
#include "table_merge.hpp"
#include "path_pass.hpp"
#include "draft.hpp"
#include "step_fused.hpp"
#include "aux_kernels.hpp"
