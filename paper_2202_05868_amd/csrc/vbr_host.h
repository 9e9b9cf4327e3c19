// Declarations shared by the host-side translation units of the library.
#pragma once

#include "vbr_internal.h"

namespace vbrk {

// Canonical-CSR check described in vbr_spmm.h; VBR_OK or VBR_EINVAL.
int validate_csr(const vbr_csr_t *csr, bool need_vals);

int sa1_reorder_impl(const vbr_csr_t *csr, int32_t col_block, double tau, int32_t *perm,
                     int32_t *row_groups, int32_t *n_groups);

// The launches one vbr_spmm call issues for dense width N, in issue order (at most VBR_MAX_LAUNCHES):
// kernel, first tile and number of tiles (or panels) of the launch, grid size.
struct Launch { int32_t kind; int32_t first_tile, n_tiles; int64_t grid; };
int plan_launches(const vbr *v, int64_t N, Launch out[VBR_MAX_LAUNCHES]);

// Thread-local code of the last failing HIP call.
void set_last_hip_error(int code);

}  // namespace vbrk
