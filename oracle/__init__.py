"""fp64 CPU oracle for the Flag Aggregator hot path.  Test infrastructure only:
imported by tests, the smoke check and the bench's cpu_baseline leg, never by the
product path."""
from .fa_oracle import (DELTA_DEFAULT, TAU_PAIR_DEFAULT, as_f64_matrix, basis_products,
                        decode_bf16, fa_literal, fa_literal_grouped, fa_scaled, multi_krum,
                        projector_difference, tsqr_r)

__all__ = ["DELTA_DEFAULT", "TAU_PAIR_DEFAULT", "as_f64_matrix", "basis_products", "decode_bf16",
           "fa_literal", "fa_literal_grouped", "fa_scaled", "multi_krum", "projector_difference",
           "tsqr_r"]
