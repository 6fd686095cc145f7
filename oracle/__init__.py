"""CPU oracle of the RRAttention prefill path: test infrastructure, never imported by the product."""
