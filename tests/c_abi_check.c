/* Compiled as plain C99 by tests/test_abi.py: the header must be usable from C, and the entry points must
 * reject bad arguments on the host (no GPU is touched: the context is NULL). */
#include <stdio.h>
#include <string.h>

#include "ais.h"

int main(void) {
  ais_params p;
  int fails = 0;
  float fake[4];
  long long cu[3] = {0, 2, 4};
  ais_params_default(&p);
  if (p.C != 5.0f || p.delta != 0.02f || p.gamma != 1.2f || p.clip_eps != 0.2f || p.adv_mode != 0) fails++;
  if (strcmp(ais_strerror(AIS_OK), "ok") != 0) fails++;
  if (ais_version() < 1000) fails++;
  if (ais_token_logprob(NULL, fake, AIS_BF16, 4, 64, 32, (const int*)fake, NULL, 1.0f, fake, fake) != AIS_ERR_STRIDE) fails++;
  if (ais_token_logprob(NULL, fake, AIS_F32, 4, 64, 64, (const int*)fake, NULL, 1.0f, fake, fake) != AIS_ERR_NULL) fails++;
  p.C = 0.5f;
  if (ais_diagnostics(NULL, fake, fake, NULL, 4, cu, 2, 2, fake, &p, fake, (int*)fake, (ais_diag*)fake) != AIS_ERR_PARAM) fails++;
  if (ais_lm_head_logprob(NULL, fake, 64, fake, 64, AIS_F32, 4, 64, 100, (const int*)fake, NULL, 1.0f, fake, fake) != AIS_ERR_DTYPE) fails++;
  if (ais_lm_head_logprob(NULL, fake, 64, fake, 64, AIS_BF16, 4, 60, 100, (const int*)fake, NULL, 1.0f, fake, fake) != AIS_ERR_SIZE) fails++;
  if (ais_destroy(NULL) != AIS_OK) fails++;
  if (sizeof(ais_diag) != 136 || sizeof(ais_params) != 40) fails++;
  printf("%d\n", fails);
  return fails;
}
