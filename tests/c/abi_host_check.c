/* The header must be plain C: this file is compiled with gcc -std=c99 -pedantic -Wall -Werror,
 * linked against libpard2cat.so and run without a GPU.  It checks the descriptor layout the
 * binding assumes and the host-only entry points (no compute call is made). */
#include <stddef.h>
#include <stdio.h>
#include <string.h>

#include "pard2_cat.h"

#define EXPECT(cond)                                              \
  do {                                                            \
    if (!(cond)) {                                                \
      fprintf(stderr, "line %d: %s is false\n", __LINE__, #cond); \
      return 1;                                                   \
    }                                                             \
  } while (0)

int main(void) {
  pard2_cat_desc d;
  pard2_kd_teacher te;
  EXPECT(sizeof(pard2_cat_desc) == 64);
  EXPECT(offsetof(pard2_cat_desc, beta) == 32);
  EXPECT(offsetof(pard2_cat_desc, ldH) == 48);
  EXPECT(offsetof(pard2_cat_desc, ldW) == 56);
  EXPECT(sizeof(pard2_kd_teacher) == 40);
  EXPECT(offsetof(pard2_kd_teacher, d) == 32);

  memset(&d, 0, sizeof d);
  d.T = 8192; d.d = 2048; d.V = 128256; d.B = 1024; d.K = 8;
  d.dtype = PARD2_BF16; d.weight_mode = PARD2_W_CAT; d.reduction = PARD2_RED_MEAN_VALID;
  d.beta = 0.1f; d.gamma = 1.0f; d.ignore_index = -100; d.ldH = 2048; d.ldW = 2048;
  EXPECT(pard2_cat_abi_version() == 1);
  EXPECT(pard2_cat_validate(&d) == PARD2_OK);
  EXPECT(pard2_cat_workspace_bytes(&d) > 0);
  EXPECT(pard2_cat_kd_workspace_bytes(&d, 4096) >= pard2_cat_workspace_bytes(&d));
  d.K = 7;
  EXPECT(pard2_cat_validate(&d) == PARD2_ERR_SHAPE);
  EXPECT(pard2_cat_workspace_bytes(&d) == 0);
  d.K = 8;
  EXPECT(pard2_cat_validate(NULL) == PARD2_ERR_NULL);
  EXPECT(strcmp(pard2_status_string(PARD2_OK), "ok") == 0);

  /* null data pointers are refused before anything is launched */
  EXPECT(pard2_cat_fwd(&d, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL, 0,
                       NULL) == PARD2_ERR_NULL);
  memset(&te, 0, sizeof te);
  te.d = 4096; te.ldH = 4096; te.ldW = 4096;
  EXPECT(pard2_cat_kd_fwd(&d, NULL, NULL, &te, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL,
                          NULL, NULL, NULL, 0, NULL) == PARD2_ERR_NULL);
  EXPECT(pard2_inject_fwd(64, 60, 32, 3, NULL, NULL, 32, NULL, NULL, NULL, NULL) == PARD2_ERR_SHAPE);
  puts("abi_host_check ok");
  return 0;
}
