/* CPU oracle (test infrastructure): declarations shared by the oracle's own
 * translation units.  Not used by the product. */
#ifndef ORACLE_INTERNAL_H
#define ORACLE_INTERNAL_H
#include "sjd_oracle.h"

#include <stddef.h>

typedef struct {
    double *k, *v;    /* [layer][position][n_kv_heads * hd] */
    size_t row;       /* n_kv_heads * hd */
    size_t per_layer; /* row * max_ctx */
    int len;          /* committed positions */
} oracle_cache;

oracle_cache *oracle_cache_new(const oracle_model_desc *md);
void oracle_cache_free(oracle_cache *c);
int oracle_forward(const oracle_model_desc *md, const oracle_weights *w, oracle_cache *cache,
                   const int32_t *tokens, int n, float *logits);
#endif
