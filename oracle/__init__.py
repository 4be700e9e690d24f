"""CPU oracle (test infrastructure only): see rago_oracle.c.  Nothing in the product path imports this."""
from .oracle import (adc_f32_topk, build, coarse, expand_pq4, flat_search, ivfpq_search, lut_f32, num_threads, quantise,
                     scan_topk, select, select_tree)
