/* A plain C99 caller of the library: the header must compile as C, every entry point must link,
 * and the host-side argument checks must answer without a GPU. */
#include "hook_api.h"

#include <stdio.h>
#include <string.h>

int main(void) {
  hook_attn_probe_args a;
  hook_capture_qk_args c;
  hook_kv_write_args w;
  hook_reduce_args r;
  int32_t layers[8], heads[8], count = 0, mode = -1;
  int fails = 0;
  memset(&a, 0, sizeof a);
  memset(&c, 0, sizeof c);
  memset(&w, 0, sizeof w);
  memset(&r, 0, sizeof r);

  fails += hook_version() < 2;
  fails += strcmp(hook_status_string(HOOK_OK), "ok") != 0;
  fails += hook_attn_probe(NULL) != HOOK_ERR_NULL;
  fails += hook_attn_probe(&a) != HOOK_ERR_SHAPE;          /* zero heads */
  fails += hook_attn_probe_workspace_bytes(&a) != 0;
  fails += hook_attn_probe_static(NULL) != HOOK_ERR_NULL;
  fails += hook_attn_probe_static(&a) != HOOK_ERR_SHAPE;   /* the same argument checks, before anything else */
  fails += hook_attn_probe_static_capacity() != HOOK_STATIC_SCRATCH_BYTES;
  a.kv_dtype = HOOK_KV_FP8_E4M3;                           /* the fields of the 8-bit cache and of the */
  a.k_scale = a.v_scale = NULL;                            /* in-call cache write are part of the struct */
  a.k_new = a.v_new = NULL;
  fails += hook_attn_probe(&a) != HOOK_ERR_SHAPE;          /* still rejected for its shapes first */
  a.kv_dtype = HOOK_KV_SAME;
  fails += hook_attn_probe_validate(NULL, &count) != HOOK_ERR_NULL;
  fails += hook_span_mass(NULL) != HOOK_ERR_NULL;
  fails += hook_span_mass_workspace_bytes(NULL) != 0;
  fails += hook_capture_qk(NULL) != HOOK_ERR_NULL;
  fails += hook_kv_write(NULL) != HOOK_ERR_NULL;
  fails += hook_reduce_mass(NULL) != HOOK_ERR_NULL;
  fails += hook_steer(NULL, NULL, 1.0f, NULL, 0, 64, HOOK_BF16, NULL) != HOOK_OK;   /* no rows: nothing to do */
  fails += hook_residual_add_steer(NULL, NULL, NULL, 1.0f, NULL, 0, 64, HOOK_BF16, NULL) != HOOK_OK;
  fails += hook_parse_layer_heads("0:0,3,6;15:2", layers, heads, 8, &count) != HOOK_OK || count != 4 ||
           layers[3] != 15 || heads[3] != 2 || heads[1] != 3;
  fails += hook_parse_config_json("{\"params\": {\"important_heads\": [[1, 2]]}, \"hookq\": {\"hookq_mode\": "
                                  "\"all_tokens\"}}", layers, heads, 8, &count, &mode) != HOOK_OK ||
           count != 1 || layers[0] != 1 || heads[0] != 2 || mode != 1;
  printf("c_abi_client: %d failure(s)\n", fails);
  return fails;
}
