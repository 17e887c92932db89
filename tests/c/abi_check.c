/* Plain-C consumer of the library's header: proves that the header is valid C99, that the
 * structs have the layout the Python binding assumes, and that the host-only entry points can be
 * called from C.  Built and run by tests/test_abi_host.py (no GPU needed). */
#include <stddef.h>
#include <stdio.h>
#include <string.h>

#include "aeris_winattn.h"

int main(void) {
  aeris_winattn_params p;
  aeris_rope_params r;
  int rc;
  memset(&p, 0, sizeof p);
  p.B = 1; p.H_lat = 64; p.W_lon = 128; p.heads = 4; p.head_dim = 32;
  p.win_h = 8; p.win_w = 8; p.shift_h = 4; p.shift_w = 4;
  p.mask_policy = AERIS_MASK_SWIN; p.out_dtype = AERIS_DT_BF16;
  r.base = 100.0f; r.positions = AERIS_ROPE_POS_GRID;
  printf("sizeof_params %zu\n", sizeof p);
  printf("offset_strides %zu\n", offsetof(aeris_winattn_params, qkv_tok_stride));
  printf("sizeof_rope %zu\n", sizeof r);
  printf("version %d\n", aeris_winattn_version());
  rc = aeris_winattn_validate(&p);
  printf("validate %d\n", rc);
  p.win_w = 7;
  printf("validate_bad %d %s\n", aeris_winattn_validate(&p), aeris_winattn_strerror(aeris_winattn_validate(&p)));
  p.win_w = 8;
  printf("bwd_ws %zu\n", aeris_winattn_bwd_workspace_bytes(&p));
  printf("rope_fwd_ws %zu\n", aeris_winattn_rope_fwd_workspace_bytes(&p));
  /* argument errors are reported before anything touches a device */
  printf("null_fwd %d\n", aeris_winattn_fwd(&p, NULL, NULL, NULL, NULL, NULL, NULL));
  printf("null_rope %d\n", aeris_rope2d_apply(&p, &r, NULL, NULL, 0, NULL));
  return 0;
}
